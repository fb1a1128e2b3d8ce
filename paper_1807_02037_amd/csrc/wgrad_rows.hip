// Weight gradient of 1x1 (1x1x1) convolutions: dw[c][k] = sum over output positions of x[pos * stride][c] * dy[pos][k].
//
// Both operands lie position-major with channels contiguous (with a stride, the rows of x are gathered), and the reduction runs over positions, so a
// work-group streams blocks of 64 positions of both tensors through LDS exactly as they lie in memory and
// reads the MFMA operands (8 consecutive positions per lane) with the gfx950 LDS transpose read.  The kernel
// is bound by the one pass over x and dy, so a work-group keeps a wide filter tile (256 x 64, 64 x 256 or
// 128 x 128 channels): with the tile covering all channels of the narrower tensor each operand is read once.
// Eight waves share a tile (two per SIMD), two register sets keep the loads of two position blocks in flight
// and LDS is double-buffered, so one barrier per block remains.  Each work-group reduces a contiguous range
// of positions and writes one partial filter; the caller sums the partials in a fixed order.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int RT = 512;      // threads per work-group
constexpr int PB = 64;       // positions per block

struct WRowsP {
  const uint16_t* X;
  const uint16_t* DY;
  float* part;
  long long rows;
  int cx, ky;
  int ctiles, ktiles, splits;
  int rows_per_split;        // multiple of PB
  int asp[3], osp[3], stride[3];   // strided variant: x is gathered at output position * stride
  // gathered-dy variant (weight gradient of a transposed convolution with window = stride): rows run over the
  // positions of x (extents asp), column j of the virtual dy is channel j % kk of tap j / kk, read at the output
  // position (extents osp) x-position * stride + tap
  int kk;
  // column sums of dy on the side (plain and strided variants): partial sums [split][ky], written by the
  // work-groups of the first channel tile of x; the caller adds them over the splits
  float* cs_part;
};

enum { ROWS_PLAIN = 0, ROWS_STRIDED_X = 1, ROWS_GATHERED_DY = 2 };

__device__ __forceinline__ bf16x8 tr_frag8(const uint16_t* p0, const uint16_t* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p0);
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p1);
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

template <int TC, int TK>
struct RowsTile {
  // a wave owns SC x SK channels of the tile: 2048 filter entries, two 32 x 32 MFMA tiles
  static constexpr int SC = TC >= 256 ? 32 : (TC == 128 ? 32 : 64);
  static constexpr int SK = 2048 / SC;
  static_assert((TC / SC) * (TK / SK) == 8, "eight waves");
  // row pitch: a 64-byte shift per row spreads the four rows of a transpose read over all banks
  static constexpr int LA = TC + 32, LB = TK + 32;
  static constexpr int XV = PB * (TC / 8) / RT, YV = PB * (TK / 8) / RT;
  static constexpr int BUF = PB * (LA + LB);                 // elements per LDS buffer
  static constexpr int LDS_BYTES = 2 * BUF * 2;
};

// Sum of the eight bf16 values of a vector into eight fp32 accumulators.
__device__ __forceinline__ void add_bf16x8(float (&acc)[8], const uint4& q) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] += __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
}

// CS: the work-groups of channel tile 0 of x also add up the rows of dy they stage (every row of dy passes through
// exactly one of them per column tile): the bias / shift gradient without another pass over dy.
template <int TC, int TK, int MODE, bool CS>
__global__ __launch_bounds__(RT, 1) void wgrad_rows_kernel(WRowsP p) {
  constexpr bool STRIDED = MODE == ROWS_STRIDED_X;
  static_assert(!CS || MODE != ROWS_GATHERED_DY, "column sums are kept for the plain and strided variants only");
  typedef RowsTile<TC, TK> T;
  constexpr int XV = T::XV, YV = T::YV, LA = T::LA, LB = T::LB;
  constexpr int FA = T::SC / 32, FB = T::SK / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_rows[];

  int b = blockIdx.x;
  const int ct = b % p.ctiles; b /= p.ctiles;
  const int kt = b % p.ktiles; b /= p.ktiles;
  const int split = b;
  const int c0 = ct * TC, k0 = kt * TK;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wc = (wave % (TC / T::SC)) * T::SC, wk = (wave / (TC / T::SC)) * T::SK;
  const int li = lane & 15, lg = lane >> 4;
  const int half = lg >> 1;
  const int src_a = (8 * half + (li >> 2)) * LA + wc + 16 * (lg & 1) + 4 * (li & 3);
  const int src_b = (8 * half + (li >> 2)) * LB + wk + 16 * (lg & 1) + 4 * (li & 3);

  const long long lo = (long long)split * p.rows_per_split;
  const long long hi = lo + p.rows_per_split < p.rows ? lo + p.rows_per_split : p.rows;
  const int nblk = hi > lo ? (int)((hi - lo + PB - 1) / PB) : 0;

  // this thread's vectors of a block: row and channel of each
  int xr[XV], xoff[XV], yr[YV], yoff[YV];
  bool xok[XV], yok[YV];
#pragma unroll
  for (int j = 0; j < XV; ++j) {
    const int v = tid + j * RT;
    xr[j] = v / (TC / 8);
    const int ch = (v % (TC / 8)) * 8;
    xok[j] = c0 + ch < p.cx;
    xoff[j] = xr[j] * p.cx + c0 + ch;
  }
#pragma unroll
  for (int j = 0; j < YV; ++j) {
    const int v = tid + j * RT;
    yr[j] = v / (TK / 8);
    const int ch = (v % (TK / 8)) * 8;
    yok[j] = k0 + ch < p.ky;
    yoff[j] = yr[j] * p.ky + k0 + ch;
    if (MODE == ROWS_GATHERED_DY) {
      // the column lies in one tap (kk is a multiple of 8): offset of the tap within the output grid, in elements
      const int col = k0 + ch;
      int t = yok[j] ? col / p.kk : 0;
      const int cc = yok[j] ? col - t * p.kk : 0;
      const int tw = t % p.stride[2]; t /= p.stride[2];
      const int th = t % p.stride[1];
      const int td = t / p.stride[1];
      yoff[j] = ((td * p.osp[1] + th) * p.osp[2] + tw) * p.kk + cc;
    }
  }

  auto fetch = [&](int blk, uint4 (&rx)[XV], uint4 (&ry)[YV]) {
    const long long r0 = lo + (long long)blk * PB;
    const uint16_t* xb = p.X + r0 * p.cx;
    const uint16_t* yb = p.DY + r0 * p.ky;
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      rx[j] = make_uint4(0, 0, 0, 0);
      if (xok[j] && r0 + xr[j] < hi) {
        if (STRIDED) {
          unsigned t = (unsigned)(r0 + xr[j]);                 // host guarantees rows < 2^31
          const unsigned ow = t % (unsigned)p.osp[2]; t /= (unsigned)p.osp[2];
          const unsigned oh = t % (unsigned)p.osp[1]; t /= (unsigned)p.osp[1];
          const unsigned od = t % (unsigned)p.osp[0]; t /= (unsigned)p.osp[0];
          const long long src = (((long long)t * p.asp[0] + od * p.stride[0]) * p.asp[1] + oh * p.stride[1]) * p.asp[2] + ow * p.stride[2];
          rx[j] = *reinterpret_cast<const uint4*>(p.X + src * p.cx + (xoff[j] - xr[j] * p.cx));
        } else {
          rx[j] = *reinterpret_cast<const uint4*>(xb + xoff[j]);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      ry[j] = make_uint4(0, 0, 0, 0);
      if (yok[j] && r0 + yr[j] < hi) {
        if (MODE == ROWS_GATHERED_DY) {
          unsigned t = (unsigned)(r0 + yr[j]);                 // host guarantees rows < 2^31
          const unsigned w = t % (unsigned)p.asp[2]; t /= (unsigned)p.asp[2];
          const unsigned h = t % (unsigned)p.asp[1]; t /= (unsigned)p.asp[1];
          const unsigned d = t % (unsigned)p.asp[0]; t /= (unsigned)p.asp[0];
          const long long row = (((long long)t * p.osp[0] + d * p.stride[0]) * p.osp[1] + h * p.stride[1]) * p.osp[2] + w * p.stride[2];
          ry[j] = *reinterpret_cast<const uint4*>(p.DY + row * p.kk + yoff[j]);
        } else {
          ry[j] = *reinterpret_cast<const uint4*>(yb + yoff[j]);
        }
      }
    }
  };
  // every vector of this thread lies in the same 8 channels (the thread count is a multiple of the vectors per row)
  float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bool cs_on = CS && ct == 0;
  auto stage = [&](uint16_t* sX, const uint4 (&rx)[XV], const uint4 (&ry)[YV]) {
    uint16_t* sY = sX + PB * LA;
    if (cs_on) {
#pragma unroll
      for (int j = 0; j < YV; ++j) add_bf16x8(csum, ry[j]);
    }
#pragma unroll
    for (int j = 0; j < XV; ++j) {
      const int v = tid + j * RT;
      *reinterpret_cast<uint4*>(sX + (v / (TC / 8)) * LA + (v % (TC / 8)) * 8) = rx[j];
    }
#pragma unroll
    for (int j = 0; j < YV; ++j) {
      const int v = tid + j * RT;
      *reinterpret_cast<uint4*>(sY + (v / (TK / 8)) * LB + (v % (TK / 8)) * 8) = ry[j];
    }
  };

  f32x16 acc[FA][FB];
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  auto multiply = [&](const uint16_t* sX) {
    const uint16_t* sY = sX + PB * LA;
#pragma unroll
    for (int ks = 0; ks < PB / 16; ++ks) {
      bf16x8 af[FA], bfr[FB];
#pragma unroll
      for (int i = 0; i < FA; ++i) {
        const uint16_t* a = sX + ks * 16 * LA + src_a + 32 * i;
        af[i] = tr_frag8(a, a + 4 * LA);
      }
#pragma unroll
      for (int j = 0; j < FB; ++j) {
        const uint16_t* q = sY + ks * 16 * LB + src_b + 32 * j;
        bfr[j] = tr_frag8(q, q + 4 * LB);
      }
#pragma unroll
      for (int i = 0; i < FA; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };

  uint4 rxa[XV], rya[YV], rxb[XV], ryb[YV];
  uint16_t* buf0 = lds_rows;
  uint16_t* buf1 = lds_rows + T::BUF;
  if (nblk > 0) {
    fetch(0, rxa, rya);
    if (nblk > 1) fetch(1, rxb, ryb);
    stage(buf0, rxa, rya);
    if (nblk > 2) fetch(2, rxa, rya);
  }
  __syncthreads();
  for (int blk = 0; blk < nblk; blk += 2) {
    // buf0 holds block blk; set b holds block blk + 1, set a block blk + 2
    if (blk + 1 < nblk) {
      stage(buf1, rxb, ryb);
      if (blk + 3 < nblk) fetch(blk + 3, rxb, ryb);
    }
    multiply(buf0);
    __syncthreads();
    if (blk + 1 < nblk) {
      if (blk + 2 < nblk) {
        stage(buf0, rxa, rya);
        if (blk + 4 < nblk) fetch(blk + 4, rxa, rya);
      }
      multiply(buf1);
      __syncthreads();
    }
  }

  float* out = p.part + (long long)split * p.cx * p.ky;
#pragma unroll
  for (int i = 0; i < FA; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int c = c0 + wc + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int k = k0 + wk + 32 * j + (lane & 31);
        if (c < p.cx && k < p.ky) out[(long long)c * p.ky + k] = acc[i][j][v];
      }
  if (cs_on) {
    // the threads tid, tid + TK / 8, ... hold the same channels: add them in a fixed order (LDS is free: the
    // loop ended with a barrier, or never ran)
    static_assert(RT * 9 * 4 <= T::LDS_BYTES, "the column sums fit the tile buffers");
    float* sh = reinterpret_cast<float*>(lds_rows);
#pragma unroll
    for (int e = 0; e < 8; ++e) sh[tid * 9 + e] = csum[e];
    __syncthreads();
    if (tid < TK && k0 + tid < p.ky) {
      constexpr int G = TK / 8;
      float t = 0.f;
      for (int i = 0; i < RT / G; ++i) t += sh[((tid >> 3) + i * G) * 9 + (tid & 7)];
      p.cs_part[(long long)split * p.ky + k0 + tid] = t;
    }
  }
}

struct RowsPlan { int tc, tk, ctiles, ktiles, splits, rows_per_split; };

RowsPlan rows_plan(long long rows, int cx, int ky) {
  // tile shape with the least traffic: x is read once per k-tile, dy once per c-tile
  static const int shapes[3][2] = {{128, 128}, {256, 64}, {64, 256}};
  RowsPlan best{};
  long long best_cost = -1;
  for (const auto& sh : shapes) {
    const int ct = (cx + sh[0] - 1) / sh[0], kt = (ky + sh[1] - 1) / sh[1];
    const long long cost = (long long)cx * kt + (long long)ky * ct;
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = RowsPlan{sh[0], sh[1], ct, kt, 0, 0}; }
  }
  long long target = 256;                                    // one work-group of eight waves per CU
  if (const char* e = getenv("LMS_WGRAD_ROWS_WGS")) target = atoll(e);
  const long long tiles = (long long)best.ctiles * best.ktiles;
  long long splits = (target + tiles - 1) / tiles;
  const long long blocks = (rows + PB - 1) / PB;
  if (splits > blocks) splits = blocks;
  if (splits < 1) splits = 1;
  const long long per = ((blocks + splits - 1) / splits) * PB;
  best.rows_per_split = (int)per;
  best.splits = (int)((rows + per - 1) / per);
  if (best.splits < 1) best.splits = 1;
  return best;
}

template <int TC, int TK, int MODE, bool CS>
hipError_t launch_rows_t(const WRowsP& p, hipStream_t s) {
  typedef RowsTile<TC, TK> T;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_rows_kernel<TC, TK, MODE, CS>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((wgrad_rows_kernel<TC, TK, MODE, CS>), dim3((unsigned)(p.ctiles * p.ktiles * p.splits)), dim3(RT), T::LDS_BYTES, s, p);
  return hipGetLastError();
}
template <int TC, int TK>
hipError_t launch_rows(const WRowsP& p, int mode, hipStream_t s) {
  if (mode == ROWS_GATHERED_DY) return launch_rows_t<TC, TK, ROWS_GATHERED_DY, false>(p, s);
  if (p.cs_part)
    return mode == ROWS_STRIDED_X ? launch_rows_t<TC, TK, ROWS_STRIDED_X, true>(p, s) : launch_rows_t<TC, TK, ROWS_PLAIN, true>(p, s);
  return mode == ROWS_STRIDED_X ? launch_rows_t<TC, TK, ROWS_STRIDED_X, false>(p, s) : launch_rows_t<TC, TK, ROWS_PLAIN, false>(p, s);
}

}  // namespace

bool wgrad_rows_eligible(int cx, int ky, const int* filt, const int* stride, const int* pad) {
  if (getenv("LMS_NO_WGRAD_ROWS")) return false;
  for (int i = 0; i < 3; ++i)
    if (filt[i] != 1 || stride[i] < 1 || pad[i] != 0) return false;
  return (cx & 7) == 0 && (ky & 7) == 0 && cx >= 48 && ky >= 48;
}

int wgrad_rows_splits(long long rows, int cx, int ky) { return rows_plan(rows, cx, ky).splits; }

hipError_t launch_wgrad_rows(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int ky, const int* asp,
                             const int* osp, const int* stride, float* cs_part, hipStream_t s) {
  const RowsPlan pl = rows_plan(rows, cx, ky);
  if ((long long)pl.ctiles * pl.ktiles * pl.splits > 0x7fffff00LL || rows >= 0x7fffff00LL) return hipErrorInvalidValue;
  if ((long long)PB * (cx > ky ? cx : ky) > 0x7fffffffLL) return hipErrorInvalidValue;     // 32-bit offsets within a block
  WRowsP p{};
  p.X = X; p.DY = DY; p.part = part; p.rows = rows; p.cx = cx; p.ky = ky; p.cs_part = cs_part;
  p.ctiles = pl.ctiles; p.ktiles = pl.ktiles; p.splits = pl.splits; p.rows_per_split = pl.rows_per_split;
  bool strided = false;
  for (int i = 0; i < 3; ++i) {
    p.asp[i] = asp[i]; p.osp[i] = osp[i]; p.stride[i] = stride[i];
    strided = strided || stride[i] != 1;
  }
  const int mode = strided ? ROWS_STRIDED_X : ROWS_PLAIN;
  if (pl.tc == 256) return launch_rows<256, 64>(p, mode, s);
  if (pl.tc == 64) return launch_rows<64, 256>(p, mode, s);
  return launch_rows<128, 128>(p, mode, s);
}

// Weight gradient of a transposed convolution whose window equals its stride (1 or 2 per axis): every output
// position belongs to one tap, so dw[t][c][k] = sum over x-positions m of x[m][c] * dy[stride * m + t][k] is a
// pointwise weight gradient whose second operand has taps * kk virtual channels.  Partial results are
// [split][c][taps * kk]; the caller sums them into [t][c][k].
bool wgrad_rows_tconv_eligible(int cx, int kk, const int* filt, const int* stride) {
  if (getenv("LMS_NO_WGRAD_ROWS")) return false;
  long long taps = 1;
  for (int i = 0; i < 3; ++i) {
    if (filt[i] != stride[i] || stride[i] < 1 || stride[i] > 2) return false;
    taps *= filt[i];
  }
  return (cx & 7) == 0 && (kk & 7) == 0 && cx >= 48 && taps * kk >= 48;
}

hipError_t launch_wgrad_rows_tconv(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int kk, const int* asp,
                                   const int* osp, const int* stride, hipStream_t s) {
  const int ky = stride[0] * stride[1] * stride[2] * kk;
  const RowsPlan pl = rows_plan(rows, cx, ky);
  if ((long long)pl.ctiles * pl.ktiles * pl.splits > 0x7fffff00LL || rows >= 0x7fffff00LL) return hipErrorInvalidValue;
  if ((long long)PB * (cx > ky ? cx : ky) > 0x7fffffffLL) return hipErrorInvalidValue;     // 32-bit offsets within a block
  if ((long long)osp[1] * osp[2] * 2 * kk > 0x7fffffffLL) return hipErrorInvalidValue;      // 32-bit tap offsets
  WRowsP p{};
  p.X = X; p.DY = DY; p.part = part; p.rows = rows; p.cx = cx; p.ky = ky; p.kk = kk;
  p.ctiles = pl.ctiles; p.ktiles = pl.ktiles; p.splits = pl.splits; p.rows_per_split = pl.rows_per_split;
  for (int i = 0; i < 3; ++i) { p.asp[i] = asp[i]; p.osp[i] = osp[i]; p.stride[i] = stride[i]; }
  if (pl.tc == 256) return launch_rows<256, 64>(p, ROWS_GATHERED_DY, s);
  if (pl.tc == 64) return launch_rows<64, 256>(p, ROWS_GATHERED_DY, s);
  return launch_rows<128, 128>(p, ROWS_GATHERED_DY, s);
}

}  // namespace lms
