// Shared by the two kernels for layers with 1 to 4 input channels (conv_small.hip, wgrad_small.hip): building the
// transposed patch matrix P^T[j][u] of 64 consecutive output positions u of one output row, j = (tap, channel).
//
// The input elements a segment needs lie in filt[0] * filt[1] input rows, contiguous within each row.  They are
// copied to LDS with loads that are contiguous across lanes (zeros where the row or the element lies outside the
// image: the padding), and P^T is then gathered out of LDS: one 2-byte LDS read and write per element instead of
// one strided 2-byte global load.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lms {
namespace {

constexpr int SG_ROWS = 64;            // positions per segment
constexpr int SG_RAWP = 512;           // elements per staged input row at most
constexpr int SG_RMAX = 16;            // staged input rows (filt[0] * filt[1]) at most
constexpr int SG_RAW_EL = (SG_RMAX + 1) * SG_RAWP;   // the staged rows and one row of zeros (read by the rows beyond J)

// Host and device: does the geometry fit the staging buffers?
inline bool sg_fits(const int* asp, const int* filt, const int* stride, int cx) {
  const long long img_bytes = 2LL * asp[0] * asp[1] * asp[2] * cx;   // one image: the range of the buffer descriptor
  return img_bytes < (1LL << 31) && filt[0] * filt[1] <= SG_RMAX && ((SG_ROWS - 1) * stride[2] + filt[2]) * cx <= SG_RAWP;
}

// code[i] = offset, in the staged rows, of element (tap, channel) j = wave + 4 i of position u = 0; the row of
// zeros beyond J.
template <int NJ>
__device__ __forceinline__ void sg_codes(int (&code)[NJ], int J, int cx, const int* filt) {
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NJ; ++i) {
    const int j = wave + 4 * i;
    const int c = j % cx;
    int t = j / cx;
    const int kw = t % filt[2]; t /= filt[2];          // t = kd * filt[1] + kh: the staged row
    code[i] = j < J ? t * SG_RAWP + kw * cx + c : SG_RMAX * SG_RAWP;
  }
}

// Staged rows of a wave: rows r = wave + 4 i, i < SG_RMAX / 4, as filter coordinates (kd, kh).
struct SgRows { int kd[SG_RMAX / 4], kh[SG_RMAX / 4]; };
__device__ __forceinline__ void sg_rows_init(SgRows& rw, const int* filt) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
  for (int i = 0; i < SG_RMAX / 4; ++i) {
    rw.kd[i] = (wave + 4 * i) / filt[1];
    rw.kh[i] = (wave + 4 * i) - rw.kd[i] * filt[1];
  }
}

// The input rows of a segment (batch nb, output row (od, oh), positions ow0 ..) go to raw[row][element] in two steps,
// so that a kernel can have the loads of the next segment in flight while it works on this one: sg_load_rows issues
// the loads into registers (a wave takes every fourth row, a lane every 64th element) through a buffer descriptor
// over the image, whose out-of-range offset returns the zeros of the padding; sg_store_rows writes the registers to
// LDS.  Which rows and elements exist is the same for the whole wave: no lane masks are kept.
// NH: loads per lane and row (64 NH elements cover a staged row).
template <int NH>
struct SgRegs { uint16_t v[SG_RMAX / 4][NH]; };

template <int NH>
__device__ __forceinline__ void sg_load_rows(SgRegs<NH>& r, const uint16_t* X, const SgRows& rw, long long nb, int od, int oh, int ow0,
                                             const int* asp, const int* stride, const int* pad, const int* filt, int cx) {
  constexpr int NI = SG_RMAX / 4;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int e_lo = (ow0 * stride[2] - pad[2]) * cx;                  // element of the image row at staged index 0
  const int row_el = asp[2] * cx;
  const int rows = filt[0] * filt[1];
  const long long img_el = (long long)asp[0] * asp[1] * row_el;
  const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(X + nb * img_el), 0, (int)(img_el * 2), 0x00020000);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    if (wave + 4 * i < rows) {
      const int id = od * stride[0] + rw.kd[i] - pad[0], ih = oh * stride[1] + rw.kh[i] - pad[1];
      const bool row_ok = (unsigned)id < (unsigned)asp[0] && (unsigned)ih < (unsigned)asp[1];
      // an absent row reads at an offset beyond the image
      const unsigned rbase = row_ok ? (unsigned)((id * asp[1] + ih) * row_el) * 2u : 0x80000000u;
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const int e = e_lo + lane + 64 * h;
        const unsigned off = (unsigned)e < (unsigned)row_el ? rbase + (unsigned)e * 2u : 0x80000000u;
        r.v[i][h] = __builtin_amdgcn_raw_buffer_load_b16(rsrc, (int)off, 0, 0);
      }
    }
  }
}

template <int NH>
__device__ __forceinline__ void sg_store_rows(uint16_t* raw, const SgRegs<NH>& r, const int* filt) {
  constexpr int NI = SG_RMAX / 4;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rows = filt[0] * filt[1];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    if (wave + 4 * i < rows) {
#pragma unroll
      for (int h = 0; h < NH; ++h) raw[(wave + 4 * i) * SG_RAWP + lane + 64 * h] = r.v[i][h];
    }
  }
}

// P^T rows j = wave + 4 i, i < NJ, of the segment; lane = position.  ustep = stride[2] * cx.  All LDS reads are
// issued before the first write.
template <int NJ>
__device__ __forceinline__ void sg_build_pt(uint16_t* sP, int pitch, const uint16_t* raw, const int (&code)[NJ], int ustep) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* src = raw + lane * ustep;
  uint16_t* dst = sP + wave * pitch + lane;
  uint16_t v[NJ];
#pragma unroll
  for (int i = 0; i < NJ; ++i) v[i] = src[code[i]];
#pragma unroll
  for (int i = 0; i < NJ; ++i) dst[4 * i * pitch] = v[i];
}

// Loads per lane and row a geometry needs, rounded to the instantiated values (2, 4, 8).
inline int sg_loads(const int* filt, const int* stride, int cx) {
  const int nh = (((SG_ROWS - 1) * stride[2] + filt[2]) * cx + 63) / 64;
  return nh <= 2 ? 2 : (nh <= 4 ? 4 : 8);
}

}  // namespace
}  // namespace lms
