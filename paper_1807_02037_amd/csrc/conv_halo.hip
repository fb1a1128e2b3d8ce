// Patch-tiled implicit-GEMM convolution for 3x3 and 3x3x3 filters with stride 1 (forward and data gradient).
//
// A work-group computes a spatial patch of 64 to 256 output positions (2-D: 8x8, 8x16 or 16x16; 3-D: 4x4x8 or 4x8x8)
// for 64 or 32 output channels.  For every block of 32 reduction channels the input patch with its one-pixel halo is
// brought into LDS once and all 9 / 27 filter taps read it from there at shifted addresses, instead of being
// gathered from global memory once per tap.  The filter is streamed through a ring of three LDS buffers, three taps
// (one filter row) per stage, requested two stages ahead, so there is one barrier per 3 taps x 32 channels of MFMA
// work and no wait for the L2 inside a stage.  The data gradient is the same computation with the taps mirrored.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

constexpr int G_TAPS = 3;      // filter taps per LDS stage (one row of the filter)

template <int P3D, int BM>
struct Patch {
  // 128 positions: 2-D 8x16, 3-D 4x4x8; 256 positions: 2-D 16x16, 3-D 4x8x8; 64 positions (2-D only, small feature maps): 8x8
  static constexpr int TD = P3D ? 4 : 1, TH = P3D ? (BM == 256 ? 8 : 4) : (BM == 256 ? 16 : 8), TW = (P3D || BM == 64) ? 8 : 16;
  static constexpr int HH = TH + 2, HW = TW + 2;                               // filters are 3 wide and high
  static constexpr int MAXPIX = (TD + (P3D ? 2 : 0)) * HH * HW;                // halo pixels at most
};

struct HaloP {
  IgemmP g;
  int flip;                // data gradient: taps mirrored
  int org[3];              // source coordinate of halo index 0 relative to the patch origin
  int hd, hh, hw;          // halo extents
  int tiles[3];            // patches per axis
  int ntiles_n;
  int ntiles;
  int batch;
};

// LDS layout and loads.
//
// A halo pixel takes 64 bytes of LDS (one block of 32 channels = four 16-byte slots); channel slot g of pixel
// (jh, jw) is stored at slot g ^ swizzle(jh, jw), chosen so that the 16 lanes a 16-byte LDS read serves per cycle
// (8 consecutive positions of two halo rows, or 16 of one) hit 16 different bank groups without any padding.  The
// filter stage (three taps x BN rows x 32 channels, 64 bytes per row, slot g ^ ((row >> 2) & 3)) is brought in
// with 16-byte buffer loads that write LDS directly (the lane's LDS address is the wave's base + 16 * lane; lanes
// whose offset lies outside the filter write zeros), two stages ahead of its use in a ring of three buffers: no
// registers, no LDS store instructions and no wait for an L2 round trip inside a stage.

typedef __attribute__((address_space(3))) void* lds_ptr_t;
// LDS address of a pointer into a __shared__ array: the low half of its generic address.
__device__ __forceinline__ lds_ptr_t lds_at(const void* p) { return (lds_ptr_t)(uint32_t)(uintptr_t)p; }

template <int TW>
__device__ __forceinline__ int halo_swizzle(int jh, int jw) {
  return TW == 8 ? (((jh & 1) << 1) | ((jw >> 2) & 1)) : ((jw >> 2) & 3);
}

// s_waitcnt vmcnt(n) only (the other counters at their maximum): at most n of this wave's memory loads, the
// LDS-direct ones included, may still be in flight.
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

template <int N>
__device__ __forceinline__ void wait_vmem() {
  static_assert(N >= 0 && N < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// PK (2-D, 8 x 16 patches): feature maps at most 7 wide and 8 high.  A patch holds two images side by side, image g of
// the pair in columns 8 g .. 8 g + 6; column 7 (and 15) stays zero and is the padding between them, to the left of the
// second image as much as to the right of the first, so every tap reads what it would read in each image alone.  Twice
// the positions per filter stage of the 8 x 8 patches that small maps otherwise take, at the same fill.
template <int P3D, int BM, int BN, int WM, int WN, int FLIP, bool PK = false>
__global__ __launch_bounds__(NTHREADS, 2) void conv_halo_kernel(HaloP hp) {
  typedef Patch<P3D, BM> PT;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int PIXB = 64;                                              // bytes per halo pixel
  constexpr int A_BYTES = PT::MAXPIX * PIXB;
  constexpr int AV = (PT::MAXPIX * 4 + NTHREADS - 1) / NTHREADS;        // halo vectors per thread
  constexpr int BV = (G_TAPS * BN * 4 + NTHREADS - 1) / NTHREADS;       // filter vectors per thread per stage
  constexpr int B_STAGE = BV * NTHREADS * 16;                           // bytes of one stage buffer (whole rounds of the work-group)
  constexpr int NBUF = 3;
  constexpr int KD = P3D ? 3 : 1;
  constexpr int NSTAGE = 3 * KD;                                        // filter rows per channel block
  static_assert(NSTAGE % NBUF == 0, "the buffer of a stage must not depend on the channel block");
  __shared__ __attribute__((aligned(16))) unsigned char smem[A_BYTES + NBUF * B_STAGE];
  unsigned char* sA = smem;
  unsigned char* sB = smem + A_BYTES;
  const IgemmP& p = hp.g;

  const int per_xcd = (hp.ntiles + 7) / 8;
  int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= hp.ntiles) return;
  const int tile_n = tile % hp.ntiles_n; tile /= hp.ntiles_n;
  const int tw = tile % hp.tiles[2]; tile /= hp.tiles[2];
  const int th = tile % hp.tiles[1]; tile /= hp.tiles[1];
  const int td = tile % hp.tiles[0]; tile /= hp.tiles[0];
  const int nb = PK ? 2 * tile : tile;                   // batch index (PK: of the first image of the pair)
  const int o0[3] = {td * PT::TD, th * PT::TH, tw * PT::TW};
  const int n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int half = lane >> 5;

  // ---- halo vectors of this thread: global element offset (or -1 = zero) and LDS byte address ----
  const int halo_pix = hp.hd * PT::HH * PT::HW;
  const int h0[3] = {o0[0] + hp.org[0], o0[1] + hp.org[1], o0[2] + hp.org[2]};
  const long long a_base = ((((long long)nb * p.asp[0] + h0[0]) * p.asp[1] + h0[1]) * p.asp[2] + h0[2]) * p.red;
  int a_off[AV];
  int a_lds[AV];
#pragma unroll
  for (int j = 0; j < AV; ++j) {
    const int v = tid + j * NTHREADS;
    const int pix = v >> 2;
    const int jw = pix % PT::HW, jh = (pix / PT::HW) % PT::HH, jd = pix / (PT::HW * PT::HH);
    const int id = h0[0] + jd, ih = h0[1] + jh, iw = h0[2] + jw;
    bool ok = pix < halo_pix && (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] &&
              (unsigned)iw < (unsigned)p.asp[2];
    a_off[j] = ok ? ((jd * p.asp[1] + jh) * p.asp[2] + jw) * p.red + (v & 3) * 8 : -1;
    if (PK) {                                  // iw is the column of the pair: image iw / 8, its column iw % 8
      const int g = iw >= 8, x = iw - 8 * g;
      ok = pix < halo_pix && (unsigned)ih < (unsigned)p.asp[1] && iw >= 0 && iw < PT::TW && x < p.asp[2] && nb + g < hp.batch;
      a_off[j] = ok ? ((g * p.asp[1] + jh) * p.asp[2] + x - h0[2]) * p.red + (v & 3) * 8 : -1;
    }
    a_lds[j] = pix * PIXB + (((v & 3) ^ halo_swizzle<PT::TW>(jh, jw)) << 4);
  }
  // ---- filter vectors of this thread within a stage: LDS slot v of the stage buffer holds row v >> 2 (tap in stage,
  // output channel), channel slot (v & 3) ^ ((row >> 2) & 3); byte offset in the filter, or out of range = zeros ----
  constexpr unsigned OOB = 0x80000000u;
  unsigned b_voff[BV];
  int b_g8[BV];
#pragma unroll
  for (int j = 0; j < BV; ++j) {
    const int v = tid + j * NTHREADS;
    const int row = v >> 2, n = row % BN, tl = row / BN;
    const int g = (v & 3) ^ ((n >> 2) & 3);
    b_g8[j] = g * 8;
    b_voff[j] = (tl < G_TAPS && n0 + n < p.nout) ? (unsigned)(((tl * p.nout + n0 + n) * p.red + g * 8) * 2) : OOB;
  }
  const __amdgpu_buffer_rsrc_t rs_b =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.B), 0, (int)((long long)p.taps * p.nout * p.red * 2), 0x00020000);
  // ---- LDS read addresses.  Operand row of tile i: position (pd, ph, pw) of the patch; tap (jd, jh, jw) reads halo
  // pixel (pd + jd, ph + jh, pw + jw), channel slot (2 ks + half) ^ swizzle.  a_rd[i][jw][x]: x = ks for 16-wide
  // patches, ks ^ (jh & 1) for 8-wide ones (the row parity is part of their swizzle). ----
  int a_rd[TM][3][2];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = wm * WTM + i * 32 + (lane & 31);
    const int pw = m % PT::TW, ph = (m / PT::TW) % PT::TH, pd = m / (PT::TW * PT::TH);
#pragma unroll
    for (int jw = 0; jw < 3; ++jw)
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int sw = halo_swizzle<PT::TW>(PT::TW == 8 ? ph : 0, pw + jw);
        a_rd[i][jw][x] = ((pd * PT::HH + ph) * PT::HW + pw + jw) * PIXB + (((x * 2 + half) ^ sw) << 4);
      }
  }
  int b_rd[TN][2];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = wn * WTN + j * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) b_rd[j][ks] = n * 64 + (((ks * 2 + half) ^ ((n >> 2) & 3)) << 4);
  }

  const int nchunks = (p.red + BK - 1) / BK;
  const int nstages = nchunks * NSTAGE;
  const unsigned b_group_bytes = (unsigned)G_TAPS * p.nout * p.red * 2;

  uint4 ra[AV];
  auto fetch_a = [&](int chunk) {
#pragma unroll
    for (int j = 0; j < AV; ++j) {
      const int c = chunk * BK + ((tid + j * NTHREADS) & 3) * 8;
      if (a_off[j] >= 0 && c < p.red) ra[j] = *reinterpret_cast<const uint4*>(p.A + a_base + a_off[j] + chunk * BK);
      else ra[j] = make_uint4(0, 0, 0, 0);
    }
  };
  // filter row `grp` of channel block `chunk` into ring buffer `buf` (all compile-time but the chunk)
  auto fetch_b = [&](int chunk, int grp, int buf) {
    const unsigned soff = (unsigned)grp * b_group_bytes + (unsigned)chunk * (BK * 2);
#pragma unroll
    for (int j = 0; j < BV; ++j) {
      const unsigned vo = (chunk * BK + b_g8[j] < p.red) ? b_voff[j] : OOB;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_b, lds_at(sB + buf * B_STAGE + (wave * 64 + j * NTHREADS) * 16), 16, vo, soff, 0, 0);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  fetch_a(0);
  fetch_b(0, 0, 0);
  fetch_b(0, 1, 1);

  const bool vec_ok = (p.nout & 7) == 0;

  for (int chunk = 0; chunk < nchunks; ++chunk) {
    const bool more = chunk + 1 < nchunks;
    auto stage = [&](auto sg_c) {                  // filter row sg = kd * 3 + kh of this channel block
      constexpr int sg = decltype(sg_c)::value;
      constexpr int kd = sg / 3, u = sg % 3;
      constexpr int buf = sg % NBUF;
      if (sg == 0) {
        __syncthreads();                       // every wave is done reading the previous channel block
#pragma unroll
        for (int j = 0; j < AV; ++j)
          if (((tid + j * NTHREADS) >> 2) < PT::MAXPIX) *reinterpret_cast<uint4*>(sA + a_lds[j]) = ra[j];
      }
      const int jd = FLIP ? KD - 1 - kd : kd;
      const int jh = FLIP ? 2 - u : u;
      const int row_off = (jd * PT::HH + jh) * PT::HW * PIXB;
      const unsigned char* b = sB + buf * B_STAGE;
      constexpr int NSTEP = G_TAPS * (BK / 16);
      constexpr int DEPTH = 2;                   // operands are read from LDS this many steps ahead of their products
      bf16x8 af[DEPTH + 1][TM], bfr[DEPTH + 1][TN];
      auto load_a = [&](int st) {
        const int tl = st / (BK / 16), ks = st % (BK / 16);
        const int jw = FLIP ? G_TAPS - 1 - tl : tl;
        const int x = PT::TW == 8 ? (ks ^ (jh & 1)) : ks;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[st % (DEPTH + 1)][i] = *reinterpret_cast<const bf16x8*>(sA + a_rd[i][jw][x] + row_off);
      };
      auto load_b = [&](int st) {
        const int tl = st / (BK / 16), ks = st % (BK / 16);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[st % (DEPTH + 1)][j] = *reinterpret_cast<const bf16x8*>(b + b_rd[j][ks] + tl * BN * 64);
      };
      // the halo does not change within a channel block: its first fragments are requested before the wait for the
      // filter stage, so that the products can start right after the barrier
      if (sg != 0) {
#pragma unroll
        for (int st = 0; st < DEPTH; ++st) load_a(st);
      }
      // this stage's filter rows have landed: every load older than the newest BV ones (and, one and two stages after
      // the halo of the next channel block was requested, those AV loads) has finished
      if (chunk * NSTAGE + sg == nstages - 1) wait_vmem<0>();          // nothing newer was requested
      else if (more && (sg == 1 || sg == 2)) wait_vmem<BV + AV>();
      else wait_vmem<BV>();
      __syncthreads();
      {   // two stages ahead: a later row of this channel block or a row of the next one
        int fg = sg + 2, fc = chunk;
        if (fg >= NSTAGE) { fg -= NSTAGE; ++fc; }
        if (fc * NSTAGE + fg < nstages) fetch_b(fc, fg, (sg + 2) % NBUF);
      }
      if (sg == 0 && more) fetch_a(chunk + 1);
      if (sg == 0) {
#pragma unroll
        for (int st = 0; st < DEPTH; ++st) load_a(st);
      }
#pragma unroll
      for (int st = 0; st < DEPTH; ++st) load_b(st);
#pragma unroll
      for (int st = 0; st < NSTEP; ++st) {
        if (st + DEPTH < NSTEP) { load_a(st + DEPTH); load_b(st + DEPTH); }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[st % (DEPTH + 1)][j], af[st % (DEPTH + 1)][i], acc[i][j], 0, 0, 0);
      }
      // pin the interleaving: the reads issued after the barrier, then per step the reads of step st + DEPTH followed
      // by the products of step st
      __builtin_amdgcn_sched_group_barrier(0x100, (sg == 0 ? TM * DEPTH : 0) + TN * DEPTH, 0);
#pragma unroll
      for (int st = 0; st < NSTEP; ++st) {
        if (st + DEPTH < NSTEP) __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
      }
    };
    static_for<NSTAGE>(stage);
  }
  __syncthreads();

  // ---- epilogue: the products were taken transposed (filter rows as the first operand), so a lane holds 16
  // output channels of one position: 4 consecutive ones per group of 4 accumulator registers, the two half-waves
  // interleaved in steps of 4.  One cross-half swap per register pair leaves 8 consecutive channels in a lane,
  // which go out as one 16-byte vector: no trip through LDS. ----
  EpiCoef coef[TN][2];
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const int n = n0 + wn * WTN + j * 32 + pr * 16 + (lane >> 5) * 8;
      if (n < p.nout) epilogue_coef(p, n, (p.nout - n) < 8 ? (p.nout - n) : 8, coef[j][pr]);
    }
  uint4 outw[TM][TN][2];
  long long pos_off[TM];
  bool pos_ok[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int r = wm * WTM + i * 32 + (lane & 31);
    const int pw = r % PT::TW, ph = (r / PT::TW) % PT::TH, pd = r / (PT::TW * PT::TH);
    const int od = o0[0] + pd, oh = o0[1] + ph, ow = o0[2] + pw;
    pos_ok[i] = od < p.osp[0] && oh < p.osp[1] && ow < p.osp[2];
    pos_off[i] = ((((long long)nb * p.osp[0] + od) * p.osp[1] + oh) * p.osp[2] + ow) * p.nout;
    if (PK) {
      const int g = pw >= 8, x = pw - 8 * g;
      pos_ok[i] = oh < p.osp[1] && x < p.osp[2] && nb + g < hp.batch;
      pos_off[i] = ((((long long)nb + g) * p.osp[1] + oh) * p.osp[2] + x) * p.nout;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][8 * pr + e]),
                                                           __float_as_uint(acc[i][j][8 * pr + 4 + e]), false, false);
          v[e] = __uint_as_float(sw[0]);
          v[4 + e] = __uint_as_float(sw[1]);
        }
        const int n = n0 + wn * WTN + j * 32 + pr * 16 + (lane >> 5) * 8;
        outw[i][j][pr] = make_uint4(0, 0, 0, 0);
        if (!pos_ok[i] || n >= p.nout) continue;
        const long long off = pos_off[i] + n;
        const int cnt = (p.nout - n) < 8 ? (p.nout - n) : 8;
        uint4 addq = make_uint4(0, 0, 0, 0), maskq = make_uint4(0, 0, 0, 0);
        if (vec_ok) {
          if (p.add) addq = *reinterpret_cast<const uint4*>(p.add + off);
          if (p.mask) maskq = *reinterpret_cast<const uint4*>(p.mask + off);
        } else {
          uint32_t aw[4] = {0, 0, 0, 0}, mw[4] = {0, 0, 0, 0};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (e < cnt) {
              if (p.add) aw[e >> 1] |= (uint32_t)p.add[off + e] << ((e & 1) * 16);
              if (p.mask) mw[e >> 1] |= (uint32_t)p.mask[off + e] << ((e & 1) * 16);
            }
          }
          addq = make_uint4(aw[0], aw[1], aw[2], aw[3]);
          maskq = make_uint4(mw[0], mw[1], mw[2], mw[3]);
        }
        outw[i][j][pr] = epilogue_pack8(p, coef[j][pr], v, addq, maskq);
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int n = n0 + wn * WTN + j * 32 + pr * 16 + (lane >> 5) * 8;
        if (pos_ok[i] && n < p.nout) epilogue_put8(p, outw[i][j][pr], (p.nout - n) < 8 ? (p.nout - n) : 8, pos_off[i] + n, vec_ok);
      }
}

template <int P3D, int BM, int BN, int WM, int WN, int FLIP, bool PK = false>
hipError_t launch_halo_t(HaloP& hp, hipStream_t s) {
  typedef Patch<P3D, BM> PT;
  const IgemmP& p = hp.g;
  hp.tiles[0] = (p.osp[0] + PT::TD - 1) / PT::TD;
  hp.tiles[1] = (p.osp[1] + PT::TH - 1) / PT::TH;
  hp.tiles[2] = (p.osp[2] + PT::TW - 1) / PT::TW;
  hp.hd = PT::TD + p.filt[0] - 1;
  hp.hh = PT::TH + p.filt[1] - 1;
  hp.hw = PT::TW + p.filt[2] - 1;
  hp.ntiles_n = (p.nout + BN - 1) / BN;
  const long long batch = p.M / ((long long)p.osp[0] * p.osp[1] * p.osp[2]);
  hp.batch = (int)batch;
  const long long nt = (PK ? (batch + 1) / 2 : batch * hp.tiles[0] * hp.tiles[1] * hp.tiles[2]) * hp.ntiles_n;
  if (nt > 0x7fffff00LL) return hipErrorInvalidValue;
  hp.ntiles = (int)nt;
  const int grid = 8 * ((hp.ntiles + 7) / 8);
  hipLaunchKernelGGL((conv_halo_kernel<P3D, BM, BN, WM, WN, FLIP, PK>), dim3(grid), dim3(NTHREADS), 0, s, hp);
  return hipGetLastError();
}

}  // namespace

// Fraction of the patch grid that covers real output positions.
static double patch_use(const IgemmP& p, int td, int th, int tw) {
  double u = 1.0;
  const int t[3] = {td, th, tw};
  for (int i = 0; i < 3; ++i) u *= (double)p.osp[i] / (double)(((p.osp[i] + t[i] - 1) / t[i]) * t[i]);
  return u;
}

bool halo_eligible(const IgemmP& p) {
  if (p.small || (p.mode != 0 && p.mode != 1)) return false;
  for (int i = 0; i < 3; ++i)
    if (p.stride[i] != 1 || (p.filt[i] != 1 && p.filt[i] != 3)) return false;
  if (p.filt[2] != 3 || p.filt[1] != 3) return false;          // stages are rows of three taps
  if ((p.red & 7) != 0) return false;
  // small feature maps fill patches badly: leave them to the row-tiled kernel
  const bool p3d = p.filt[0] == 3;
  return (p3d ? patch_use(p, 4, 4, 8) : std::max(patch_use(p, 1, 8, 16), patch_use(p, 1, 8, 8))) >= 0.6;
}

template <int P3D, int FLIP>
static hipError_t launch_halo_pf(HaloP& hp, hipStream_t s) {
  const IgemmP& p = hp.g;
  static const int force_bm = getenv("LMS_HALO_BM") ? atoi(getenv("LMS_HALO_BM")) : 0;   // tuning aid
  const double u128 = P3D ? patch_use(p, 4, 4, 8) : patch_use(p, 1, 8, 16);
  const double u256 = P3D ? patch_use(p, 4, 8, 8) : patch_use(p, 1, 16, 16);
  bool big = u256 >= 0.9 * u128 && p.M >= 256 * 1024;     // enough patches to fill the chip with the larger tile
  if (force_bm) big = force_bm == 256;
  const bool narrow = p.nout <= 32;
  // maps at most 7 wide and 8 high of a same-size convolution: two images per 8x16 patch
  static const bool no_pairs = getenv("LMS_NO_HALO_PAIRS") != nullptr;   // tuning aid
  if constexpr (!P3D) {
    if (!no_pairs && !force_bm && !narrow && p.osp[2] <= 7 && p.osp[1] <= 8 && p.asp[1] == p.osp[1] && p.asp[2] == p.osp[2] &&
        hp.org[2] == -1 && p.M >= 2LL * p.osp[1] * p.osp[2])
      return launch_halo_t<0, 128, 64, 2, 2, FLIP, true>(hp, s);
  }
  // small 2-D feature maps (7x7): 8x8 patches, 64 positions per work-group, fill the chip and the patches better
  if (!P3D && !force_bm && !narrow && patch_use(p, 1, 8, 8) > 1.25 * u128) return launch_halo_t<P3D, 64, 64, 2, 2, FLIP>(hp, s);
  if (big) return narrow ? launch_halo_t<P3D, 256, 32, 4, 1, FLIP>(hp, s) : launch_halo_t<P3D, 256, 64, 4, 1, FLIP>(hp, s);
  return narrow ? launch_halo_t<P3D, 128, 32, 4, 1, FLIP>(hp, s) : launch_halo_t<P3D, 128, 64, 2, 2, FLIP>(hp, s);
}

hipError_t launch_halo(IgemmP& p, hipStream_t s) {
  HaloP hp{};
  hp.g = p;
  hp.flip = p.mode == 1;
  for (int i = 0; i < 3; ++i) hp.org[i] = p.mode == 0 ? -p.pad[i] : p.pad[i] - (p.filt[i] - 1);
  const bool p3d = p.filt[0] == 3;
  if (hp.flip) return p3d ? launch_halo_pf<1, 1>(hp, s) : launch_halo_pf<0, 1>(hp, s);
  return p3d ? launch_halo_pf<1, 0>(hp, s) : launch_halo_pf<0, 0>(hp, s);
}

}  // namespace lms
