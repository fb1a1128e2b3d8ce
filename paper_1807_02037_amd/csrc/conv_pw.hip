// Pointwise (1x1 / 1x1x1, stride 1, no padding) forward convolution:
//   out[m][k] = epi(sum_c x[m][c] * w[c][k]),  m over positions, channels-last rows.
//
// Without filter taps the operation is a plain GEMM whose long side is the position count, and with the
// channel counts of CNN bottlenecks it is bound by the one pass over the activations.  This kernel stages
// 128 positions x 64 input channels per step with contiguous 16-byte loads and keeps the filter in the
// layout it has in memory ([c][k]): the filter tile is stored [c][k] in LDS and the MFMA operand (8 consecutive
// c per lane) is read with the gfx950 LDS transpose read, so no filter repacking kernel runs before it.
// LDS is double-buffered (one barrier per stage); the epilogue (scale/shift, residual add, ReLU) is the
// shared 8-channel vector epilogue.  (The data gradient of a pointwise convolution reads the filter along
// its contiguous axis already and stays on the general kernel, which measured faster for it.)
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int PM = 128;       // positions per tile
constexpr int PK = 64;        // reduction channels per stage
constexpr int PLA = PK + 8;   // pitch of [row][r] tiles (144 bytes: conflict-free 16-byte reads)

template <int BN>
struct PwTile {
  static constexpr int LBT = BN + 32;                       // pitch of the [r][n] filter tile (64-byte row shift)
  static constexpr int A_EL = PM * PLA;
  static constexpr int B_EL = PK * LBT;
  static constexpr int STAGE = A_EL + B_EL;
  static constexpr int LDC = BN + 4;
  static constexpr int MAIN_BYTES = 2 * STAGE * 2, EPI_BYTES = PM * LDC * 4;
  static constexpr int LDS_BYTES = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
};

__device__ __forceinline__ bf16x8 pw_tr_frag(const uint16_t* p0, const uint16_t* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p0);
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p1);
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// UP: the transposed-convolution variant (one product per tap parity, output rows remapped); a template parameter so
// that the plain pointwise kernel keeps its 32-bit tile-relative addressing.
template <int BN, bool UP>
__global__ __launch_bounds__(NTHREADS, (BN == 64 ? 3 : 2)) void pw_kernel(IgemmP p) {
  typedef PwTile<BN> T;
  constexpr int TN = BN / 32;
  constexpr int AV = PM * (PK / 8) / NTHREADS;                              // 4 activation vectors per thread
  constexpr int BV = PK * (BN / 8) / NTHREADS;                              // filter vectors per thread
  constexpr int LDC = T::LDC;
  extern __shared__ __attribute__((aligned(16))) unsigned char pw_smem[];
  uint16_t* sA = reinterpret_cast<uint16_t*>(pw_smem);
  float* sC = reinterpret_cast<float*>(pw_smem);

  const int per_xcd = (p.ntiles + 7) / 8;
  int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= p.ntiles) return;
  // Transposed convolution with window = stride: every output position takes one filter tap (the parity of its
  // coordinates), so the layer is one pointwise product of the input with taps x k virtual output channels: column
  // n is channel n % k of tap n / k, filter element w[tap][c][n % k], written to the output position
  // stride * input position + tap.  The input tile is read once for all taps of a column tile, and the taps that
  // differ in the last coordinate only are neighbours in memory, so their channels leave as one contiguous run.
  const int npar = UP ? p.up[0] * p.up[1] * p.up[2] : 1;
  const int nv = npar * p.nout;                           // virtual output channels
  const int n0 = (tile % p.ntiles_n) * BN;
  const long long m0 = (long long)(tile / p.ntiles_n) * PM;
  const uint16_t* Bp = p.B;
  // element offset, in the output tensor, of column n of input row m (UP only)
  auto out_off = [&](long long m, int n) -> long long {
    int t = n / p.nout;
    const int kk = n - t * p.nout;
    const int tw = t % p.up[2]; t /= p.up[2];
    const int th = t % p.up[1];
    const int td = t / p.up[1];
    const int w = (int)(m % p.asp[2]); long long q = m / p.asp[2];
    const int h = (int)(q % p.asp[1]); q /= p.asp[1];
    const int d = (int)(q % p.asp[0]); q /= p.asp[0];
    return (((q * p.osp[0] + d * p.up[0] + td) * p.osp[1] + h * p.up[1] + th) * p.osp[2] + w * p.up[2] + tw) * (long long)p.nout + kk;
  };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  // UP: output row of tap 0 for each input row of the tile (read by the epilogue after the main loop's barriers)
  __shared__ unsigned s_row0[UP ? PM : 1];
  if (UP && tid < PM) {
    const long long m = m0 + tid < p.M ? m0 + tid : 0;
    const int w = (int)(m % p.asp[2]); long long q = m / p.asp[2];
    const int h = (int)(q % p.asp[1]); q /= p.asp[1];
    const int d = (int)(q % p.asp[0]); q /= p.asp[0];
    s_row0[tid] = (unsigned)(((q * p.osp[0] + d * p.up[0]) * p.osp[1] + h * p.up[1]) * p.osp[2] + w * p.up[2]);
  }

  // global offsets of this thread's vectors for stage 0
  long long a_off[AV];
  bool a_ok[AV];
#pragma unroll
  for (int j = 0; j < AV; ++j) {
    const int v = tid + j * NTHREADS;
    const long long m = m0 + (v >> 3);
    a_ok[j] = m < p.M;
    a_off[j] = m * p.red + (v & 7) * 8;
  }
  long long b_off[BV];
  bool b_ok[BV];
#pragma unroll
  for (int j = 0; j < BV; ++j) {
    const int v = tid + j * NTHREADS;
    const int r = v / (BN / 8), col = (v % (BN / 8)) * 8;
    b_ok[j] = n0 + col < nv;
    b_off[j] = (long long)r * p.nout + n0 + col;
    if (UP) {                                             // column of tap t: w[t][r][kk]
      const int t = (n0 + col) / p.nout;
      b_off[j] = ((long long)t * p.red + r) * p.nout + (n0 + col - t * p.nout);
    }
  }
  const int niter = (p.red + PK - 1) / PK;

  uint4 ra[AV], rb[BV];
  auto load_stage = [&](int it) {
    const int k0 = it * PK;
#pragma unroll
    for (int j = 0; j < AV; ++j) {
      const int cv = ((tid + j * NTHREADS) & 7) * 8;
      ra[j] = make_uint4(0, 0, 0, 0);
      if (a_ok[j] && k0 + cv < p.red) ra[j] = *reinterpret_cast<const uint4*>(p.A + a_off[j] + k0);
    }
#pragma unroll
    for (int j = 0; j < BV; ++j) {
      const int v = tid + j * NTHREADS;
      rb[j] = make_uint4(0, 0, 0, 0);
      const int r = v / (BN / 8);
      if (b_ok[j] && k0 + r < p.red) rb[j] = *reinterpret_cast<const uint4*>(Bp + b_off[j] + (long long)k0 * p.nout);
    }
  };
  auto store_stage = [&](int buf) {
    uint16_t* a = sA + buf * T::STAGE;
    uint16_t* b = a + T::A_EL;
#pragma unroll
    for (int j = 0; j < AV; ++j) {
      const int v = tid + j * NTHREADS;
      *reinterpret_cast<uint4*>(a + (v >> 3) * PLA + (v & 7) * 8) = ra[j];
    }
#pragma unroll
    for (int j = 0; j < BV; ++j) {
      const int v = tid + j * NTHREADS;
      *reinterpret_cast<uint4*>(b + (v / (BN / 8)) * T::LBT + (v % (BN / 8)) * 8) = rb[j];
    }
  };

  f32x16 acc[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

  load_stage(0);

  // operands of the epilogue do not depend on the main loop: fetch them now
  constexpr int EV = PM * (BN / 8) / NTHREADS;
  uint4 pre_add[EV], pre_mask[EV];
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    pre_add[q] = make_uint4(0, 0, 0, 0);
    pre_mask[q] = make_uint4(0, 0, 0, 0);
    const int idx = tid + q * NTHREADS;
    const int r = idx / (BN / 8), cg = (idx % (BN / 8)) * 8;
    if (m0 + r < p.M && n0 + cg < nv && (!UP || p.add || p.mask)) {
      const long long off = UP ? out_off(m0 + r, n0 + cg) : m0 * p.nout + n0 + (unsigned)(r * p.nout + cg);
      if (p.add) pre_add[q] = *reinterpret_cast<const uint4*>(p.add + off);
      if (p.mask) pre_mask[q] = *reinterpret_cast<const uint4*>(p.mask + off);
    }
  }

  const long long tile_base = m0 * p.nout + n0;
  store_stage(0);
  __syncthreads();
  for (int it = 0; it < niter; ++it) {
    if (it + 1 < niter) load_stage(it + 1);
    const uint16_t* a = sA + (it & 1) * T::STAGE;
    const uint16_t* b = a + T::A_EL;
#pragma unroll
    for (int ks = 0; ks < PK / 16; ++ks) {
      const bf16x8 af = *reinterpret_cast<const bf16x8*>(a + (wave * 32 + (lane & 31)) * PLA + ks * 16 + (lane >> 5) * 8);
      bf16x8 bfr[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const uint16_t* q = b + (ks * 16 + 8 * (lg >> 1) + (li >> 2)) * T::LBT + 32 * j + 16 * (lg & 1) + 4 * (li & 3);
        bfr[j] = pw_tr_frag(q, q + 4 * T::LBT);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr[j], acc[j], 0, 0, 0);
    }
    if (it + 1 < niter) store_stage((it + 1) & 1);
    __syncthreads();
  }

  // epilogue: accumulators -> LDS (row-major fp32) -> 8-channel vectors
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wave * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      sC[row * LDC + j * 32 + (lane & 31)] = acc[j][v];
    }
  __syncthreads();
  // every vector of this thread has the same channels (the thread count is a multiple of the vectors per row)
  const int cg = (tid % (BN / 8)) * 8, n = n0 + cg;
  EpiCoef coef;
  if (n < nv) epilogue_coef(p, UP ? n % p.nout : n, 8, coef);
  // UP: this thread's columns lie in one tap: its row offset in the output grid and the channel within the tap
  long long up_tap_row = 0;
  int up_kk = 0;
  if (UP && n < nv) {
    int t = n / p.nout;
    up_kk = n - t * p.nout;
    const int tw = t % p.up[2]; t /= p.up[2];
    const int th = t % p.up[1];
    const int td = t / p.up[1];
    up_tap_row = ((long long)td * p.osp[1] + th) * p.osp[2] + tw;
  }
  uint4 outw[EV];
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    const int r = (tid + q * NTHREADS) / (BN / 8);
    outw[q] = make_uint4(0, 0, 0, 0);
    if (m0 + r >= p.M || n >= nv) continue;
    const float4 lo = *reinterpret_cast<const float4*>(sC + r * LDC + cg);
    const float4 hi = *reinterpret_cast<const float4*>(sC + r * LDC + cg + 4);
    const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    outw[q] = epilogue_pack8(p, coef, v, pre_add[q], pre_mask[q]);
  }
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    const int r = (tid + q * NTHREADS) / (BN / 8);
    if (m0 + r < p.M && n < nv)
      epilogue_put8(p, outw[q], 8, UP ? ((long long)s_row0[r] + up_tap_row) * p.nout + up_kk : tile_base + (unsigned)(r * p.nout + cg), true);
  }
}

template <int BN, bool UP>
hipError_t launch_pw_t(IgemmP& p, hipStream_t s) {
  typedef PwTile<BN> T;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(pw_kernel<BN, UP>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
  if (attr != hipSuccess) return attr;
  const int npar = UP ? p.up[0] * p.up[1] * p.up[2] : 1;
  p.ntiles_n = (npar * p.nout + BN - 1) / BN;
  const long long mt = (p.M + PM - 1) / PM;
  if (mt * p.ntiles_n > 0x7fffff00LL || p.M >= 0x7fffffffLL) return hipErrorInvalidValue;
  p.ntiles = (int)(mt * p.ntiles_n);
  const int grid = 8 * ((p.ntiles + 7) / 8);
  hipLaunchKernelGGL((pw_kernel<BN, UP>), dim3(grid), dim3(NTHREADS), T::LDS_BYTES, s, p);
  return hipGetLastError();
}

}  // namespace

bool pw_eligible(const IgemmP& p) {
  static const bool off = getenv("LMS_NO_PW") != nullptr;   // tuning aid
  if (off || p.small || p.taps != 1) return false;
  for (int i = 0; i < 3; ++i)
    if (p.filt[i] != 1 || p.stride[i] != 1 || p.pad[i] != 0) return false;
  return (p.red & 7) == 0 && (p.nout & 7) == 0 && p.nout >= 32 && p.red >= 32;
}

// Transposed convolution with window = stride (1 or 2 per axis) as pointwise products, filter read as stored.
bool pw_up_eligible(const IgemmP& p) {
  static const bool off = getenv("LMS_NO_PW") != nullptr;   // tuning aid
  if (off) return false;
  for (int i = 0; i < 3; ++i)
    if (p.up[i] < 1 || p.up[i] > 2 || p.osp[i] != p.asp[i] * p.up[i]) return false;
  return (p.red & 7) == 0 && (p.nout & 7) == 0 && p.nout >= 32 && p.red >= 32;
}

hipError_t launch_pw(IgemmP& p, hipStream_t s) {
  if (p.up[0] > 0) return p.up[0] * p.up[1] * p.up[2] * p.nout <= 64 ? launch_pw_t<64, true>(p, s) : launch_pw_t<128, true>(p, s);
  return p.nout <= 64 ? launch_pw_t<64, false>(p, s) : launch_pw_t<128, false>(p, s);
}

}  // namespace lms
