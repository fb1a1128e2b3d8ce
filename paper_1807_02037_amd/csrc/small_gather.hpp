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

// Host and device: does the geometry fit the staging buffers?
inline bool sg_fits(const int* asp, const int* filt, const int* stride, int cx) {
  const long long img_bytes = 2LL * asp[0] * asp[1] * asp[2] * cx;   // one image: the range of the buffer descriptor
  return img_bytes < (1LL << 31) && filt[0] * filt[1] <= SG_RMAX && ((SG_ROWS - 1) * stride[2] + filt[2]) * cx <= SG_RAWP;
}

// code[i] = offset, in the staged rows, of element (tap, channel) j = wave + 4 i of position u = 0.
template <int NJ>
__device__ __forceinline__ void sg_codes(int (&code)[NJ], int J, int cx, const int* filt) {
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NJ; ++i) {
    const int j = wave + 4 * i;
    const int c = j % cx;
    int t = j / cx;
    const int kw = t % filt[2]; t /= filt[2];          // t = kd * filt[1] + kh: the staged row
    code[i] = j < J ? t * SG_RAWP + kw * cx + c : 0;
  }
}

// Copies the input rows of the segment (batch nb, output row (od, oh), positions ow0 ..) to raw[row][element].
// All loads are issued before the first LDS write (a load in flight per staged row and half row), through a buffer
// descriptor over the image, whose out-of-range offset returns the zeros of the padding.  256 threads.
__device__ __forceinline__ void sg_stage_rows(uint16_t* raw, const uint16_t* X, long long nb, int od, int oh, int ow0, const int* asp,
                                              const int* stride, const int* pad, const int* filt, int cx) {
  const int nel = ((SG_ROWS - 1) * stride[2] + filt[2]) * cx;        // elements per staged row
  const int e_lo = (ow0 * stride[2] - pad[2]) * cx;                  // element of the image row at staged index 0
  const int row_el = asp[2] * cx;
  const int rows = filt[0] * filt[1];
  const long long img_el = (long long)asp[0] * asp[1] * row_el;
  const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(X + nb * img_el), 0, (int)(img_el * 2), 0x00020000);
  const int tid = threadIdx.x;
  uint16_t v[SG_RMAX][2];
  int kd = 0, kh = 0;
#pragma unroll
  for (int r = 0; r < SG_RMAX; ++r) {
    if (r < rows) {
      const int id = od * stride[0] + kd - pad[0], ih = oh * stride[1] + kh - pad[1];
      const bool row_ok = (unsigned)id < (unsigned)asp[0] && (unsigned)ih < (unsigned)asp[1];
      const int rbase = (id * asp[1] + ih) * row_el;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int q = tid + h * 256;
        const int e = e_lo + q;
        const bool ok = row_ok && q < nel && (unsigned)e < (unsigned)row_el;
        const unsigned off = ok ? (unsigned)(rbase + e) * 2u : 0x80000000u;
        v[r][h] = __builtin_amdgcn_raw_buffer_load_b16(rsrc, (int)off, 0, 0);
      }
      if (++kh == filt[1]) { kh = 0; ++kd; }
    }
  }
#pragma unroll
  for (int r = 0; r < SG_RMAX; ++r) {
    if (r < rows) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int q = tid + h * 256;
        if (q < nel) raw[r * SG_RAWP + q] = v[r][h];
      }
    }
  }
}

// P^T rows j = wave, wave + 4, ... (< J) of the segment; lane = position.  ustep = stride[2] * cx.  All LDS reads
// are issued before the first write.
template <int NJ>
__device__ __forceinline__ void sg_build_pt(uint16_t* sP, int pitch, const uint16_t* raw, const int (&code)[NJ], int J, int ustep) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint16_t* src = raw + lane * ustep;
  uint16_t* dst = sP + wave * pitch + lane;
  const int ni = (J - wave + 3) >> 2;                  // rows of this wave
  uint16_t v[NJ];
#pragma unroll
  for (int i = 0; i < NJ; ++i)
    if (i < ni) v[i] = src[code[i]];
#pragma unroll
  for (int i = 0; i < NJ; ++i)
    if (i < ni) dst[4 * i * pitch] = v[i];
}

}  // namespace
}  // namespace lms
