// Types shared by the convolution kernel files (internal).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lms {

struct IgemmP {
  const uint16_t* A;
  const uint16_t* B;
  uint16_t* out;
  const float* scale;
  const float* shift;
  const uint16_t* add;
  const uint16_t* mask;
  int relu;
  long long M;
  int nout, red;
  int asp[3], osp[3], filt[3], stride[3], pad[3];
  int mode;     // 0: src = o*stride + tap - pad (forward); 1: src = (o + pad - tap)/stride (transposed)
  int taps;
  int small;    // reduction index is (tap, channel) flattened, channel count not a multiple of 8
  int jpad;     // small mode: row pitch of B, multiple of BK
  int ntiles_n;
  int ntiles;   // total tiles
  int up[3];    // pointwise kernel as a transposed convolution with window = stride: upsampling factor per axis (0: off)
  // strided transposed gather tiled by residue class: positions per class and axis, rows per class, tiles per class
  int qsp[3];
  long long Mc;
  int cls_tiles;
};

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   // keep NaN a NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                              // nearest even
  return (uint16_t)(u >> 16);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// Two floats -> two bf16 (round to nearest even) in one 32-bit word, low half first: v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

constexpr int BK = 32;        // reduction elements per stage
constexpr int LDA = BK + 8;   // LDS row pitch (bf16): 80 bytes, keeps 16-byte reads conflict-free
constexpr int NTHREADS = 256;




// Epilogue of 8-channel vectors of output rows: v = acc*scale + shift + add; ReLU; ReLU mask; bf16.  It comes in
// three pieces so that a kernel can load the per-channel coefficients once, do the arithmetic of all its vectors,
// and only then issue all stores together: a wait for a load placed between two stores would also wait for the
// older store to be acknowledged.  Which terms are present is the same for the whole launch, so each term is a
// uniform branch around a few vector instructions.
struct EpiCoef { float sc[8], sh[8]; };

// Scale and shift of the channels n .. n+7 (cnt of them exist).
__device__ __forceinline__ void epilogue_coef(const IgemmP& p, int n, int cnt, EpiCoef& c) {
#pragma unroll
  for (int e = 0; e < 8; ++e) { c.sc[e] = 1.f; c.sh[e] = 0.f; }
  if (p.scale) {
    if (cnt == 8) {
      const float4 a = *reinterpret_cast<const float4*>(p.scale + n), b = *reinterpret_cast<const float4*>(p.scale + n + 4);
      c.sc[0] = a.x; c.sc[1] = a.y; c.sc[2] = a.z; c.sc[3] = a.w; c.sc[4] = b.x; c.sc[5] = b.y; c.sc[6] = b.z; c.sc[7] = b.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e < cnt) c.sc[e] = p.scale[n + e];
    }
  }
  if (p.shift) {
    if (cnt == 8) {
      const float4 a = *reinterpret_cast<const float4*>(p.shift + n), b = *reinterpret_cast<const float4*>(p.shift + n + 4);
      c.sh[0] = a.x; c.sh[1] = a.y; c.sh[2] = a.z; c.sh[3] = a.w; c.sh[4] = b.x; c.sh[5] = b.y; c.sh[6] = b.z; c.sh[7] = b.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e < cnt) c.sh[e] = p.shift[n + e];
    }
  }
}

// The arithmetic of one vector; addq / maskq hold the eight bf16 values of the add and mask tensors (zero words if
// absent).  Returns the eight bf16 results.
__device__ __forceinline__ uint4 epilogue_pack8(const IgemmP& p, const EpiCoef& c, const float (&v)[8], const uint4& addq,
                                                const uint4& maskq) {
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = v[e];
  if (p.scale || p.shift) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(x[e], c.sc[e], c.sh[e]);
  }
  if (p.add) {
    const uint32_t addw[4] = {addq.x, addq.y, addq.z, addq.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] += __uint_as_float((e & 1) ? (addw[e >> 1] & 0xffff0000u) : (addw[e >> 1] << 16));
  }
  if (p.relu) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = __builtin_amdgcn_fmed3f(x[e], 0.f, __builtin_inff());   // one instruction; NaN -> 0 like fmaxf
  }
  if (p.mask) {
    const uint32_t maskw[4] = {maskq.x, maskq.y, maskq.z, maskq.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float mv = __uint_as_float((e & 1) ? (maskw[e >> 1] & 0xffff0000u) : (maskw[e >> 1] << 16));
      x[e] = mv > 0.f ? x[e] : 0.f;
    }
  }
  return make_uint4(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7]));
}

// Stores `cnt` (<= 8) channels at out + off; vec: the row pitch allows one 16-byte store.
__device__ __forceinline__ void epilogue_put8(const IgemmP& p, const uint4& w, int cnt, long long off, bool vec) {
  if (vec) *reinterpret_cast<uint4*>(p.out + off) = w;
  else {
    const uint32_t ow[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (e < cnt) p.out[off + e] = (uint16_t)(ow[e >> 1] >> ((e & 1) * 16));
  }
}

}  // namespace

// Patch-tiled kernel for 3x3 / 3x3x3 stride-1 filters (conv_halo.hip).
bool halo_eligible(const IgemmP& p);
hipError_t launch_halo(IgemmP& p, hipStream_t s);

// Resident-filter kernel for 2-D 3x3 64->64 and 3-D 3x3x3 32->32 channels, stride 1 (conv_rf.hip).
bool rf_eligible(const IgemmP& p);
hipError_t launch_rf(IgemmP& p, hipStream_t s);

// Patch-tiled weight gradient for 3x3 / 3x3x3 stride-1 filters (wgrad_patch.hip): writes per-split partial
// filters [split][tap][cx][ky]; the caller sums them.
bool wgrad_patch_eligible(int cx, int ky, const int* filt, const int* stride);
int wgrad_patch_splits(long long batch, const int* asp, const int* osp, const int* filt, const int* pad, int cx, int ky);
// cs_part (only where wgrad_patch_colsum says so, else null): partial column sums of dy [split][ky] on the side.
bool wgrad_patch_colsum(const int* filt, int cx, int ky);
hipError_t launch_wgrad_patch(const uint16_t* X, const uint16_t* DY, float* part, long long batch, const int* asp,
                              const int* osp, const int* filt, const int* pad, int cx, int ky, float* cs_part, hipStream_t s);

// Pointwise (1x1, stride 1) forward convolution (conv_pw.hip).  p.B is the filter as stored, [c][k].
bool pw_eligible(const IgemmP& p);
bool pw_up_eligible(const IgemmP& p);   // p.up set, p.M = input rows, p.asp / p.osp = input / output extents
hipError_t launch_pw(IgemmP& p, hipStream_t s);

// Weight gradient of a transposed convolution with window = stride on the pointwise weight-gradient kernel
// (wgrad_rows.hip): partial results [split][cx][taps * kk], splits = wgrad_rows_splits(rows, cx, taps * kk).
bool wgrad_rows_tconv_eligible(int cx, int kk, const int* filt, const int* stride);
hipError_t launch_wgrad_rows_tconv(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int kk, const int* asp,
                                   const int* osp, const int* stride, hipStream_t s);

// Forward convolution with at most 4 input channels and at most 64 output channels (conv_small.hip).  p.B is the filter as stored.
bool conv_small_eligible(const IgemmP& p);
hipError_t launch_conv_small(IgemmP& p, hipStream_t s);

// Weight gradient for convolutions with at most 4 input channels (wgrad_small.hip): per-split partial filters [split][tap][cx][ky].
bool wgrad_small_eligible(int cx, int ky, const int* asp, const int* filt, const int* stride);
int wgrad_small_splits(long long rows, const int* osp);
hipError_t launch_wgrad_small(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int ky, const int* asp,
                              const int* osp, const int* filt, const int* stride, const int* pad, hipStream_t s);

// Streaming weight gradient for 1x1 filters without padding (wgrad_rows.hip): per-split partial filters [split][cx][ky].
bool wgrad_rows_eligible(int cx, int ky, const int* filt, const int* stride, const int* pad);
int wgrad_rows_splits(long long rows, int cx, int ky);
// cs_part (or null): partial column sums of dy [split][ky] on the side.
hipError_t launch_wgrad_rows(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int ky, const int* asp,
                             const int* osp, const int* stride, float* cs_part, hipStream_t s);

}  // namespace lms
