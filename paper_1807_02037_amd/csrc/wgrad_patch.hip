// Weight gradient of 3x3 / 3x3x3 stride-1 convolutions, patch-tiled.
//
// A work-group owns 32 input channels x 32 output channels of the filter gradient and walks over a
// range of spatial patches (128 output positions: 2-D 8x16, 3-D 4x4x8).  Per patch it brings the input
// patch with its halo (32 channels) and the output-gradient patch (32 channels) into LDS exactly as they
// lie in memory (position-major, channels contiguous); every filter tap is then a row offset into the
// same input tile.  The reduction runs over positions, so the MFMA operands must hold 8 consecutive
// positions per lane: they are read with the gfx950 LDS transpose read (ds_read_b64_tr_b16), which hands
// lane i of a 16-lane group the element (i % 4) of the four 8-byte rows addressed by lanes i/4, i/4+4,
// i/4+8, i/4+12 (layout checked on the device).  The 9 / 27 taps are dealt to the four waves; each wave
// keeps one 32x32 accumulator per tap.  Partial gradients per work-group go to the split buffer and are
// summed in a fixed order by the reduction kernel.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

struct WPatchP {
  const uint16_t* X;
  const uint16_t* DY;
  float* part;
  int batch;
  int asp[3], osp[3], filt[3], pad[3];
  int cx, ky, taps;
  int cchunks, ktiles, splits;
  int tiles[3];
  int patches;             // batch * tiles (pairs of images in the packed form of the 64 x 64 kernel)
  int patches_per_split;
  unsigned x_bytes, y_bytes;   // tensor sizes if both are below 2 GiB (32-bit buffer offsets), else 0
  float* cs_part;              // 64 x 64 tile kernel: partial column sums of dy [split][ky] on the side, or null
};

constexpr int LDX = 32;    // LDS row pitch in bf16 elements: 64 bytes = 16 banks, so the four rows of a transpose read cover all 64 banks (no conflicts measured)

template <int P3D>
struct WPatch {
  static constexpr int TD = P3D ? 4 : 1, TH = P3D ? 4 : 8, TW = P3D ? 8 : 16;
  static constexpr int HH = TH + 2, HW = TW + 2;
  static constexpr int MAXPIX = (TD + (P3D ? 2 : 0)) * HH * HW;
  static constexpr int MAXT = P3D ? 7 : 3;          // taps per wave at most
};

__device__ __forceinline__ bf16x8 tr_frag(const uint16_t* p0, const uint16_t* p1) {
  // two transpose reads: positions 0..3 and 4..7 of this lane's half
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p0);
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p1);
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Wave w owns the contiguous taps [TAPS*w/4, TAPS*(w+1)/4).  The taps kw = 0, 1, 2 of one filter row (kd, kh) read
// the positions p .. p+9 of one halo row: where a wave has several of them, the 12 positions p .. p+11 are fetched
// once (three transpose reads) and the fragments of the three taps are cut out in registers.
template <int P3D, int W>
__device__ __forceinline__ void wgrad_patch_mma(const uint16_t* sX, const uint16_t* sY, f32x16 (&acc)[WPatch<P3D>::MAXT], int src_off,
                                                int half) {
  typedef WPatch<P3D> PT;
  constexpr int TAPS = P3D ? 27 : 9;
  constexpr int LO = TAPS * W / 4, HI = TAPS * (W + 1) / 4;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    // positions q0 .. q0+7 of this lane's half: one row (or half row) of the patch, contiguous in the halo tile
    const int q0 = ks * 16 + 8 * half;
    const int pw = q0 % PT::TW, ph = (q0 / PT::TW) % PT::TH, pd = q0 / (PT::TW * PT::TH);
    const uint16_t* xb = sX + ((pd * PT::HH + ph) * PT::HW + pw) * LDX + src_off;
    const uint16_t* yb = sY + q0 * LDX + src_off;
    const bf16x8 bfr = tr_frag(yb, yb + 4 * LDX);
#pragma unroll
    for (int row = LO / 3; row <= (HI - 1) / 3; ++row) {
      const int k_lo = (LO > row * 3 ? LO : row * 3) - row * 3, k_hi = (HI < row * 3 + 3 ? HI : row * 3 + 3) - row * 3;   // kw range
      const uint16_t* xr = xb + ((row / 3) * PT::HH + (row % 3)) * PT::HW * LDX;
      if (k_hi - k_lo == 1) {
        const bf16x8 af = tr_frag(xr + k_lo * LDX, xr + (k_lo + 4) * LDX);
        acc[row * 3 + k_lo - LO] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[row * 3 + k_lo - LO], 0, 0, 0);
      } else {
        typedef unsigned v2u __attribute__((ext_vector_type(2)));
        typedef unsigned v4u __attribute__((ext_vector_type(4)));
        const v2u r0 = __builtin_bit_cast(v2u, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)xr));
        const v2u r1 = __builtin_bit_cast(v2u, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(xr + 4 * LDX)));
        const v2u r2 = __builtin_bit_cast(v2u, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(xr + 8 * LDX)));
        const unsigned u[6] = {r0[0], r0[1], r1[0], r1[1], r2[0], r2[1]};     // two positions per word
#pragma unroll
        for (int kw = k_lo; kw < k_hi; ++kw) {
          v4u f;
          if (kw == 0) f = v4u{u[0], u[1], u[2], u[3]};
          else if (kw == 2) f = v4u{u[1], u[2], u[3], u[4]};
          else f = v4u{__builtin_amdgcn_alignbit(u[1], u[0], 16), __builtin_amdgcn_alignbit(u[2], u[1], 16),
                       __builtin_amdgcn_alignbit(u[3], u[2], 16), __builtin_amdgcn_alignbit(u[4], u[3], 16)};
          acc[row * 3 + kw - LO] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f), bfr, acc[row * 3 + kw - LO], 0, 0, 0);
        }
      }
    }
  }
}

template <int P3D>
__global__ __launch_bounds__(NTHREADS, 2) void wgrad_patch_kernel(WPatchP p) {
  typedef WPatch<P3D> PT;
  constexpr int XV = (PT::MAXPIX * 4 + NTHREADS - 1) / NTHREADS;   // input-tile vectors per thread
  constexpr int YV = 128 * 4 / NTHREADS;                           // gradient-tile vectors per thread
  __shared__ __attribute__((aligned(16))) uint16_t sX[(PT::MAXPIX + 4) * LDX];     // the 12-position reads of the last halo row run 2 pixels over
  __shared__ __attribute__((aligned(16))) uint16_t sY[128 * LDX];

  int b = blockIdx.x;
  const int cc = b % p.cchunks; b /= p.cchunks;
  const int kt = b % p.ktiles; b /= p.ktiles;
  const int split = b;
  const int c0 = cc * 32, k0 = kt * 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hd = PT::TD + p.filt[0] - 1;
  const int halo_pix = hd * PT::HH * PT::HW;

  // this lane as a source of the transpose reads: position offset i/4 within a group of four, channels 16*(g&1) + 4*(i&3)
  const int li = lane & 15, lg = lane >> 4;
  const int src_off = (li >> 2) * LDX + 16 * (lg & 1) + 4 * (li & 3);
  const int half = lg >> 1;                                   // which 8 of the 16 positions of a k-step

  // halo coordinates of this thread's input vectors (relative to the patch origin)
  int xj[XV][3];
  bool x_valid[XV];
#pragma unroll
  for (int j = 0; j < XV; ++j) {
    const int pix = (tid + j * NTHREADS) >> 2;
    x_valid[j] = pix < halo_pix;
    unsigned t = x_valid[j] ? (unsigned)pix : 0u;
    xj[j][2] = (int)(t % PT::HW); t /= PT::HW;
    xj[j][1] = (int)(t % PT::HH); t /= PT::HH;
    xj[j][0] = (int)t;
  }
  int yj[YV][3];
#pragma unroll
  for (int j = 0; j < YV; ++j) {
    const int q = (tid + j * NTHREADS) >> 2;
    yj[j][2] = q % PT::TW; yj[j][1] = (q / PT::TW) % PT::TH; yj[j][0] = q / (PT::TW * PT::TH);
  }
  const int vch = (tid & 3) * 8;                               // channel offset of this thread's vectors
  const bool xc_ok = c0 + vch < p.cx, yc_ok = k0 + vch < p.ky;
  const bool x_vec = (p.cx & 7) == 0;

  const int pbegin = split * p.patches_per_split;
  const int pend = (pbegin + p.patches_per_split < p.patches) ? pbegin + p.patches_per_split : p.patches;

  // 32-bit offsets of this thread's vectors relative to the patch origin (input: origin - pad)
  int x_rel[XV], y_rel[YV];
#pragma unroll
  for (int j = 0; j < XV; ++j) x_rel[j] = ((xj[j][0] * p.asp[1] + xj[j][1]) * p.asp[2] + xj[j][2]) * p.cx + c0 + vch;
#pragma unroll
  for (int j = 0; j < YV; ++j) y_rel[j] = ((yj[j][0] * p.osp[1] + yj[j][1]) * p.osp[2] + yj[j][2]) * p.ky + k0 + vch;

  uint4 rx[XV], ry[YV];
  // patch coordinates advance one patch at a time (no divisions in the loop)
  int tw, th, td;
  long long nb;
  {
    unsigned t = (unsigned)pbegin;
    tw = (int)(t % (unsigned)p.tiles[2]); t /= (unsigned)p.tiles[2];
    th = (int)(t % (unsigned)p.tiles[1]); t /= (unsigned)p.tiles[1];
    td = (int)(t % (unsigned)p.tiles[0]); t /= (unsigned)p.tiles[0];
    nb = t;
  }
  auto advance = [&]() {
    if (++tw == p.tiles[2]) { tw = 0; if (++th == p.tiles[1]) { th = 0; if (++td == p.tiles[0]) { td = 0; ++nb; } } }
  };
  // With 8-channel vectors and tensors below 2 GiB, memory is read through buffer descriptors: an offset beyond the
  // tensor returns zeros, so padding and ragged patches need no branches and no 64-bit address arithmetic.
  const bool use_buf = x_vec && p.x_bytes != 0;
  constexpr int OOB = (int)0x80000000;
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.X), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.DY), 0, (int)p.y_bytes, 0x00020000);
  auto fetch = [&]() {
    const int o0[3] = {td * PT::TD, th * PT::TH, tw * PT::TW};
    const int i0[3] = {o0[0] - p.pad[0], o0[1] - p.pad[1], o0[2] - p.pad[2]};
    if (use_buf) {
      const int xb = (((((int)nb * p.asp[0] + i0[0]) * p.asp[1] + i0[1]) * p.asp[2] + i0[2]) * p.cx) * 2;
      const int yb = (((((int)nb * p.osp[0] + o0[0]) * p.osp[1] + o0[1]) * p.osp[2] + o0[2]) * p.ky) * 2;
#pragma unroll
      for (int j = 0; j < XV; ++j) {
        const bool ok = x_valid[j] && xc_ok && (unsigned)(i0[0] + xj[j][0]) < (unsigned)p.asp[0] &&
                        (unsigned)(i0[1] + xj[j][1]) < (unsigned)p.asp[1] && (unsigned)(i0[2] + xj[j][2]) < (unsigned)p.asp[2];
        rx[j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, ok ? xb + 2 * x_rel[j] : OOB, 0, 0));
      }
#pragma unroll
      for (int j = 0; j < YV; ++j) {
        const bool ok = yc_ok && o0[0] + yj[j][0] < p.osp[0] && o0[1] + yj[j][1] < p.osp[1] && o0[2] + yj[j][2] < p.osp[2];
        ry[j] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_y, ok ? yb + 2 * y_rel[j] : OOB, 0, 0));
      }
      return;
    }
    const uint16_t* xb = p.X + (((nb * p.asp[0] + i0[0]) * p.asp[1] + i0[1]) * p.asp[2] + i0[2]) * p.cx;
    const uint16_t* yb = p.DY + (((nb * p.osp[0] + o0[0]) * p.osp[1] + o0[1]) * p.osp[2] + o0[2]) * p.ky;
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int id = i0[0] + xj[j][0], ih = i0[1] + xj[j][1], iw = i0[2] + xj[j][2];
      rx[j] = make_uint4(0, 0, 0, 0);
      if (x_valid[j] && xc_ok && (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] &&
          (unsigned)iw < (unsigned)p.asp[2]) {
        const uint16_t* src = xb + x_rel[j];
        if (x_vec) rx[j] = *reinterpret_cast<const uint4*>(src);
        else {        // channel count not a multiple of 8 (first layer): element by element
          uint32_t w4[4] = {0, 0, 0, 0};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (c0 + vch + e < p.cx) w4[e >> 1] |= (uint32_t)src[e] << ((e & 1) * 16);
          rx[j] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      const int od = o0[0] + yj[j][0], oh = o0[1] + yj[j][1], ow = o0[2] + yj[j][2];
      ry[j] = make_uint4(0, 0, 0, 0);
      if (yc_ok && od < p.osp[0] && oh < p.osp[1] && ow < p.osp[2]) ry[j] = *reinterpret_cast<const uint4*>(yb + y_rel[j]);
    }
  };

  f32x16 acc[PT::MAXT];
#pragma unroll
  for (int j = 0; j < PT::MAXT; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  if (pbegin < pend) fetch();
  for (int patch = pbegin; patch < pend; ++patch) {
    __syncthreads();                       // previous patch fully consumed
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int v = tid + j * NTHREADS;
      if ((v >> 2) < PT::MAXPIX) *reinterpret_cast<uint4*>(sX + (v >> 2) * LDX + (v & 3) * 8) = rx[j];
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      const int v = tid + j * NTHREADS;
      *reinterpret_cast<uint4*>(sY + (v >> 2) * LDX + (v & 3) * 8) = ry[j];
    }
    __syncthreads();
    if (patch + 1 < pend) { advance(); fetch(); }
    switch (wave) {
      case 0: wgrad_patch_mma<P3D, 0>(sX, sY, acc, src_off, half); break;
      case 1: wgrad_patch_mma<P3D, 1>(sX, sY, acc, src_off, half); break;
      case 2: wgrad_patch_mma<P3D, 2>(sX, sY, acc, src_off, half); break;
      default: wgrad_patch_mma<P3D, 3>(sX, sY, acc, src_off, half); break;
    }
  }
  const int tap_lo = p.taps * wave / 4, tap_n = p.taps * (wave + 1) / 4 - tap_lo;
#pragma unroll
  for (int j = 0; j < PT::MAXT; ++j) {
    const int t = tap_lo + j;
    if (j >= tap_n) continue;
    float* out = p.part + ((long long)split * p.taps + t) * p.cx * p.ky;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int c = c0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const int k = k0 + (lane & 31);
      if (c < p.cx && k < p.ky) out[(long long)c * p.ky + k] = acc[j][v];
    }
  }
}


// 2-D variant with a 64 x 64 channel tile per work-group: every wave owns one 32 x 32 quadrant with all nine
// taps (nine accumulators), so an input patch and a gradient patch are read from memory once for 64 x 64
// filter entries instead of once per 32 x 32.
constexpr int LDW = 72;    // LDS row pitch: 64 channels + 8 (144 bytes)
constexpr int WGRAD64_LDS_BYTES = 2 * (10 * 18 + 128) * LDW * 2;

// CS: the work-groups of input-channel tile 0 also add up the gradient vectors they stage (every position of dy
// lies in exactly one patch): the bias / shift gradient without another pass over dy.
// PK: feature maps at most 7 wide and 8 high (the last stage of ResNet-50: 7 x 7), where one image fills 49 of a
// patch's 128 positions.  A patch then holds two images side by side, image g of the pair in columns 8 g .. 8 g + 6:
// column 7 (and 15) stays zero and is the padding between them, to the left of the second image as much as to the
// right of the first, so the nine taps read what they would read in each image alone.
template <bool CS, bool PK>
__global__ __launch_bounds__(NTHREADS, 1) void wgrad_patch64_kernel(WPatchP p) {
  constexpr int TH = 8, TW = 16, HH = TH + 2, HW = TW + 2, PIX = HH * HW;
  constexpr int XV = (PIX * 8 + NTHREADS - 1) / NTHREADS;        // 6 input vectors per thread
  constexpr int YV = 128 * 8 / NTHREADS;                         // 4 gradient vectors per thread
  // two buffers of (input halo tile, gradient tile): one is multiplied while the next patch is written
  extern __shared__ __attribute__((aligned(16))) uint16_t lds64[];
  constexpr int BUF = (PIX + 128) * LDW;
  static_assert(2 * BUF * 2 == WGRAD64_LDS_BYTES, "launch passes the LDS size");

  int b = blockIdx.x;
  const int cc = b % p.cchunks; b /= p.cchunks;
  const int kt = b % p.ktiles; b /= p.ktiles;
  const int split = b;
  const int c0 = cc * 64, k0 = kt * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ch = (wave & 1) * 32, kh = (wave >> 1) * 32;       // this wave's quadrant

  const int li = lane & 15, lg = lane >> 4;
  const int src_off = (li >> 2) * LDW + 16 * (lg & 1) + 4 * (li & 3);
  const int half = lg >> 1;

  int xh[XV], xw[XV], x_rel[XV];
  bool x_valid[XV];
  const int vch = (tid & 7) * 8;
#pragma unroll
  for (int j = 0; j < XV; ++j) {
    const int pix = (tid + j * NTHREADS) >> 3;
    x_valid[j] = pix < PIX && c0 + vch < p.cx;
    const int t = pix < PIX ? pix : 0;
    xw[j] = t % HW; xh[j] = t / HW;
    x_rel[j] = (xh[j] * p.asp[2] + xw[j]) * p.cx + c0 + vch;
    if (PK) {
      const int vc = xw[j] - p.pad[2];                       // column of the pair: image vc / 8, its column vc % 8
      const int g = vc >= 8;
      xw[j] = g;                                             // from here on: which image of the pair
      x_valid[j] = x_valid[j] && vc >= 0 && vc < TW && vc - 8 * g < p.asp[2];
      x_rel[j] = ((g * p.asp[1] + xh[j]) * p.asp[2] + vc - 8 * g) * p.cx + c0 + vch;
    }
  }
  int yh[YV], yw[YV], y_rel[YV];
  const bool yc_ok = k0 + vch < p.ky;
#pragma unroll
  for (int j = 0; j < YV; ++j) {
    const int q = (tid + j * NTHREADS) >> 3;
    yw[j] = q % TW; yh[j] = q / TW;
    y_rel[j] = (yh[j] * p.osp[2] + yw[j]) * p.ky + k0 + vch;
    if (PK) {
      const int g = yw[j] >= 8, x = yw[j] - 8 * g;
      y_rel[j] = ((g * p.osp[1] + yh[j]) * p.osp[2] + x) * p.ky + k0 + vch;
      yw[j] = x < p.osp[2] ? g : 2;                          // which image of the pair; 2: the padding column
    }
  }

  const int pbegin = split * p.patches_per_split;
  const int pend = (pbegin + p.patches_per_split < p.patches) ? pbegin + p.patches_per_split : p.patches;

  uint4 rxa[XV], rya[YV];
  auto fetch = [&](int patch, uint4 (&rx)[XV], uint4 (&ry)[YV]) {
    unsigned t = (unsigned)patch;
    const int tw = (int)(t % (unsigned)p.tiles[2]); t /= (unsigned)p.tiles[2];
    const int th = (int)(t % (unsigned)p.tiles[1]); t /= (unsigned)p.tiles[1];
    const long long nb = PK ? 2LL * patch : (long long)t;       // PK: one patch per pair of images
    const int oh0 = PK ? 0 : th * TH, ow0 = PK ? 0 : tw * TW;
    const int ih0 = oh0 - p.pad[1], iw0 = PK ? 0 : ow0 - p.pad[2];
    const uint16_t* xb = p.X + ((nb * p.asp[1] + ih0) * p.asp[2] + iw0) * p.cx;
    const uint16_t* yb = p.DY + ((nb * p.osp[1] + oh0) * p.osp[2] + ow0) * p.ky;
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      rx[j] = make_uint4(0, 0, 0, 0);
      const bool col_ok = PK ? nb + xw[j] < p.batch : (unsigned)(iw0 + xw[j]) < (unsigned)p.asp[2];
      if (x_valid[j] && (unsigned)(ih0 + xh[j]) < (unsigned)p.asp[1] && col_ok)
        rx[j] = *reinterpret_cast<const uint4*>(xb + x_rel[j]);
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      ry[j] = make_uint4(0, 0, 0, 0);
      const bool col_ok = PK ? (yw[j] < 2 && nb + yw[j] < p.batch) : ow0 + yw[j] < p.osp[2];
      if (yc_ok && oh0 + yh[j] < p.osp[1] && col_ok) ry[j] = *reinterpret_cast<const uint4*>(yb + y_rel[j]);
    }
  };

  f32x16 acc[9];
#pragma unroll
  for (int j = 0; j < 9; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};     // channels k0 + vch .. + 7 of all this thread's vectors
  const bool cs_on = CS && cc == 0;
  auto stage = [&](uint16_t* sX, const uint4 (&rx)[XV], const uint4 (&ry)[YV]) {
    uint16_t* sY = sX + PIX * LDW;
    if (cs_on) {
#pragma unroll
      for (int j = 0; j < YV; ++j) {
        const uint32_t w[4] = {ry[j].x, ry[j].y, ry[j].z, ry[j].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) csum[e] += __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
      }
    }
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int v = tid + j * NTHREADS;
      if ((v >> 3) < PIX) *reinterpret_cast<uint4*>(sX + (v >> 3) * LDW + (v & 7) * 8) = rx[j];
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      const int v = tid + j * NTHREADS;
      *reinterpret_cast<uint4*>(sY + (v >> 3) * LDW + (v & 7) * 8) = ry[j];
    }
  };
  auto multiply = [&](const uint16_t* sX) {
    const uint16_t* sY = sX + PIX * LDW;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      // one k-step is one row of the patch; the tap (r, s) reads the halo tile r rows down and s columns right
      const int q0 = ks * 16 + 8 * half;
      const int pw = q0 % TW, ph = q0 / TW;
      const uint16_t* yb = sY + q0 * LDW + src_off + kh;
      const bf16x8 bfr = tr_frag(yb, yb + 4 * LDW);
      const uint16_t* xb0 = sX + (ph * HW + pw) * LDW + src_off + ch;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const uint16_t* xb = xb0 + ((t / 3) * HW + (t % 3)) * LDW;
        const bf16x8 af = tr_frag(xb, xb + 4 * LDW);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[t], 0, 0, 0);
      }
    }
  };

  if (pbegin < pend) {
    fetch(pbegin, rxa, rya);
    stage(lds64, rxa, rya);
    if (pbegin + 1 < pend) fetch(pbegin + 1, rxa, rya);
  }
  __syncthreads();
  int cur = 0;
  for (int patch = pbegin; patch < pend; ++patch) {
    if (patch + 1 < pend) {
      stage(lds64 + (cur ^ 1) * BUF, rxa, rya);          // the other buffer was last read before the barrier below
      if (patch + 2 < pend) fetch(patch + 2, rxa, rya);
    }
    multiply(lds64 + cur * BUF);
    __syncthreads();
    cur ^= 1;
  }
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    float* out = p.part + ((long long)split * 9 + t) * p.cx * p.ky;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int c = c0 + ch + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const int k = k0 + kh + (lane & 31);
      if (c < p.cx && k < p.ky) out[(long long)c * p.ky + k] = acc[t][v];
    }
  }
  if (cs_on) {
    // threads tid, tid + 8, ... hold the same channels: add them in a fixed order (the loop ended with a barrier,
    // or never ran, so LDS is free)
    float* sh = reinterpret_cast<float*>(lds64);
#pragma unroll
    for (int e = 0; e < 8; ++e) sh[tid * 9 + e] = csum[e];
    __syncthreads();
    if (tid < 64 && k0 + tid < p.ky) {
      float t = 0.f;
      for (int i = 0; i < NTHREADS / 8; ++i) t += sh[((tid >> 3) + i * 8) * 9 + (tid & 7)];
      p.cs_part[(long long)split * p.ky + k0 + tid] = t;
    }
  }
}

// 64 x 64 channel tile: 2-D filters with at least 48 channels on both sides
bool wide_tile(const int* filt, int cx, int ky) {
  if (getenv("LMS_NO_WGRAD_WIDE")) return false;
  return filt[0] == 1 && cx >= 48 && ky >= 48 && (cx & 7) == 0;
}

// Two images per patch (the PK form of the 64 x 64 kernel): same-size 3 x 3 convolution on maps at most 7 wide and 8 high.
bool pair_packed(const int* asp, const int* osp, const int* filt, const int* pad, int cx, int ky) {
  if (getenv("LMS_NO_WGRAD_PAIRS")) return false;   // tuning aid
  return wide_tile(filt, cx, ky) && osp[2] <= 7 && osp[1] <= 8 && asp[1] == osp[1] && asp[2] == osp[2] && pad[2] == 1;
}

struct PatchGrid { int tiles[3]; long long patches; int splits, per_split; bool pairs; };
PatchGrid patch_grid(long long batch, const int* asp, const int* osp, const int* filt, const int* pad, int cx, int ky) {
  PatchGrid g;
  const bool p3d = filt[0] == 3;
  const int td = p3d ? 4 : 1, th = p3d ? 4 : 8, tw = p3d ? 8 : 16;
  g.tiles[0] = (osp[0] + td - 1) / td;
  g.tiles[1] = (osp[1] + th - 1) / th;
  g.tiles[2] = (osp[2] + tw - 1) / tw;
  g.patches = batch * g.tiles[0] * g.tiles[1] * g.tiles[2];
  g.pairs = pair_packed(asp, osp, filt, pad, cx, ky);
  if (g.pairs) g.patches = (batch + 1) / 2;
  const int tile = wide_tile(filt, cx, ky) ? 64 : 32;
  const long long wg = (long long)((cx + tile - 1) / tile) * ((ky + tile - 1) / tile);
  // partial sums cost 4 bytes x filter size per work-group, written and read again: two work-groups per compute unit
  // (32 x 32 tiles) measured 5 % faster on the 3D U-Net step than four
  long long target = tile == 64 ? 256 : 512;
  if (const char* e = getenv("LMS_WGRAD_PATCH_WGS")) target = atoll(e);
  long long splits = (target + wg - 1) / wg;
  if (splits > g.patches) splits = g.patches;
  if (splits < 1) splits = 1;
  g.per_split = (int)((g.patches + splits - 1) / splits);
  g.splits = (int)((g.patches + g.per_split - 1) / g.per_split);
  return g;
}

}  // namespace

bool wgrad_patch_eligible(int cx, int ky, const int* filt, const int* stride) {
  for (int i = 0; i < 3; ++i)
    if (stride[i] != 1) return false;
  if (filt[1] != 3 || filt[2] != 3 || (filt[0] != 1 && filt[0] != 3)) return false;
  (void)cx;                       // any input channel count: odd counts are gathered element by element
  return (ky & 7) == 0;
}

int wgrad_patch_splits(long long batch, const int* asp, const int* osp, const int* filt, const int* pad, int cx, int ky) {
  return patch_grid(batch, asp, osp, filt, pad, cx, ky).splits;
}

bool wgrad_patch_colsum(const int* filt, int cx, int ky) { return wide_tile(filt, cx, ky); }

hipError_t launch_wgrad_patch(const uint16_t* X, const uint16_t* DY, float* part, long long batch, const int* asp,
                              const int* osp, const int* filt, const int* pad, int cx, int ky, float* cs_part, hipStream_t s) {
  if (cs_part && !wide_tile(filt, cx, ky)) return hipErrorInvalidValue;
  WPatchP p{};
  p.X = X; p.DY = DY; p.part = part; p.cs_part = cs_part;
  p.batch = (int)batch;
  for (int i = 0; i < 3; ++i) { p.asp[i] = asp[i]; p.osp[i] = osp[i]; p.filt[i] = filt[i]; p.pad[i] = pad[i]; }
  p.cx = cx; p.ky = ky; p.taps = filt[0] * filt[1] * filt[2];
  p.cchunks = (cx + 31) / 32; p.ktiles = (ky + 31) / 32;
  const PatchGrid g = patch_grid(batch, asp, osp, filt, pad, cx, ky);
  if (g.patches > 0x7fffff00LL) return hipErrorInvalidValue;
  for (int i = 0; i < 3; ++i) p.tiles[i] = g.tiles[i];
  p.patches = (int)g.patches; p.splits = g.splits; p.patches_per_split = g.per_split;
  const long long xb = batch * asp[0] * asp[1] * asp[2] * cx * 2, yb = batch * osp[0] * osp[1] * osp[2] * ky * 2;
  if (xb < 0x7fffff00LL && yb < 0x7fffff00LL) { p.x_bytes = (unsigned)xb; p.y_bytes = (unsigned)yb; }
  if (wide_tile(filt, cx, ky)) {
    p.cchunks = (cx + 63) / 64; p.ktiles = (ky + 63) / 64;
    auto run = [&](auto kernel) -> hipError_t {
      const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, WGRAD64_LDS_BYTES);
      if (attr != hipSuccess) return attr;
      const dim3 grid((unsigned)(p.cchunks * p.ktiles * p.splits));
      hipLaunchKernelGGL(kernel, grid, dim3(NTHREADS), WGRAD64_LDS_BYTES, s, p);
      return hipGetLastError();
    };
    if (g.pairs) return cs_part ? run(wgrad_patch64_kernel<true, true>) : run(wgrad_patch64_kernel<false, true>);
    return cs_part ? run(wgrad_patch64_kernel<true, false>) : run(wgrad_patch64_kernel<false, false>);
  }
  const long long blocks = (long long)p.cchunks * p.ktiles * p.splits;
  if (filt[0] == 3) hipLaunchKernelGGL(wgrad_patch_kernel<1>, dim3((unsigned)blocks), dim3(NTHREADS), 0, s, p);
  else hipLaunchKernelGGL(wgrad_patch_kernel<0>, dim3((unsigned)blocks), dim3(NTHREADS), 0, s, p);
  return hipGetLastError();
}

}  // namespace lms
