// Patch-tiled implicit-GEMM convolution for 3x3 and 3x3x3 filters with stride 1 (forward and data gradient).
//
// A work-group computes a spatial patch of 128 output positions (2-D: 8x16, 3-D: 4x4x8) for 64 or 32
// output channels.  For every block of 32 reduction channels the input patch with its one-pixel halo is
// brought into LDS once and all 9 / 27 filter taps read it from there at shifted addresses, instead of being
// gathered from global memory once per tap.  The filter is streamed through LDS three taps (one filter row)
// at a time, double-buffered, so there is one barrier per 3 taps x 32 channels of MFMA work.  The data
// gradient is the same computation with the filter taps mirrored.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

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
};

template <int P3D, int BM, int BN, int WM, int WN, int FLIP>
__global__ __launch_bounds__(NTHREADS, 2) void conv_halo_kernel(HaloP hp) {
  typedef Patch<P3D, BM> PT;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  // LDS pitch of a halo row.  A 16-byte read serves 16 lanes per cycle: one halo row of the 2-D patch (conflict-free
  // at the pixel pitch), but two rows of a 3-D patch (8 positions wide), whose bank sets are disjoint only if the rows
  // lie 128 bytes apart modulo 256; 10 pixels of 80 bytes are 32 modulo 256, hence 96 bytes of padding.  The 256 x 64
  // tile stays unpadded: with the padding only one work-group would fit a compute unit, which costs more.
  constexpr int ROWP = PT::HW * LDA + ((PT::TW == 8 && !(BM == 256 && BN == 64)) ? 48 : 0);
  constexpr int A_ELEMS = (PT::TD + (P3D ? 2 : 0)) * PT::HH * ROWP;
  constexpr int B_ELEMS = G_TAPS * BN * LDA;
  constexpr int MAIN_BYTES = (A_ELEMS + 2 * B_ELEMS) * 2;
  constexpr int SMEM = MAIN_BYTES;
  constexpr int AV = (PT::MAXPIX * 4 + NTHREADS - 1) / NTHREADS;     // halo vectors per thread
  constexpr int BV = (G_TAPS * BN * 4 + NTHREADS - 1) / NTHREADS;    // filter vectors per thread per stage
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  uint16_t* sA = reinterpret_cast<uint16_t*>(smem);
  uint16_t* sB = sA + A_ELEMS;
  const IgemmP& p = hp.g;

  const int per_xcd = (hp.ntiles + 7) / 8;
  int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= hp.ntiles) return;
  const int tile_n = tile % hp.ntiles_n; tile /= hp.ntiles_n;
  const int tw = tile % hp.tiles[2]; tile /= hp.tiles[2];
  const int th = tile % hp.tiles[1]; tile /= hp.tiles[1];
  const int td = tile % hp.tiles[0]; tile /= hp.tiles[0];
  const int nb = tile;                                   // batch index
  const int o0[3] = {td * PT::TD, th * PT::TH, tw * PT::TW};
  const int n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- halo vectors of this thread: element offset in A (without the channel-block offset), -1 = zero ----
  const int halo_pix = hp.hd * PT::HH * PT::HW;
  // element offset of pixel (0,0,0) of the halo, and 32-bit pixel offsets relative to it
  const int h0[3] = {o0[0] + hp.org[0], o0[1] + hp.org[1], o0[2] + hp.org[2]};
  const long long a_base = ((((long long)nb * p.asp[0] + h0[0]) * p.asp[1] + h0[1]) * p.asp[2] + h0[2]) * p.red;
  int a_off[AV];      // (pixel offset from a_base) * red + channel vector, or -1 for padding
#pragma unroll
  for (int j = 0; j < AV; ++j) {
    const int v = tid + j * NTHREADS;
    const int pix = v >> 2;
    const int jw = pix % PT::HW, jh = (pix / PT::HW) % PT::HH, jd = pix / (PT::HW * PT::HH);
    const int id = h0[0] + jd, ih = h0[1] + jh, iw = h0[2] + jw;
    const bool ok = pix < halo_pix && (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] &&
                    (unsigned)iw < (unsigned)p.asp[2];
    a_off[j] = ok ? ((jd * p.asp[1] + jh) * p.asp[2] + jw) * p.red + (v & 3) * 8 : -1;
  }
  // ---- filter vectors of this thread within a stage: (tap in stage, row n, 8-channel vector) ----
  int b_off[BV];
  bool b_ok[BV];
#pragma unroll
  for (int j = 0; j < BV; ++j) {
    const int v = tid + j * NTHREADS;
    const int cv = v & 3, n = (v >> 2) % BN, tl = (v >> 2) / BN;
    b_ok[j] = tl < G_TAPS && n0 + n < p.nout;
    b_off[j] = (tl * p.nout + n0 + n) * p.red + cv * 8;
  }
  // ---- per-lane halo pixel of the first tap for each 32-row MFMA tile of this wave ----
  int a_pix[TM];      // LDS element offset of that pixel
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = wm * WTM + i * 32 + (lane & 31);
    const int pw = m % PT::TW, ph = (m / PT::TW) % PT::TH, pd = m / (PT::TW * PT::TH);
    a_pix[i] = (pd * PT::HH + ph) * ROWP + pw * LDA;
  }

  const int nchunks = (p.red + BK - 1) / BK;
  constexpr int KD = P3D ? 3 : 1;                  // filter planes; a plane has three rows of three taps
  // filter stages are fetched RBD stages ahead (an L2 hit takes longer than one stage of MFMA work); the 2 x 2 wave
  // tile has no registers to spare for three sets
  constexpr int RBD = TM * TN < 4 ? 3 : 1;
  constexpr bool PIPE = TM * TN < 4;               // second fragment set: operands of the next step are read early
  const long long b_group_stride = (long long)G_TAPS * p.nout * p.red;

  uint4 ra[AV], rb[RBD][BV];
  auto fetch_a = [&](int chunk) {
#pragma unroll
    for (int j = 0; j < AV; ++j) {
      const int c = chunk * BK + ((tid + j * NTHREADS) & 3) * 8;
      if (a_off[j] >= 0 && c < p.red) ra[j] = *reinterpret_cast<const uint4*>(p.A + a_base + a_off[j] + chunk * BK);
      else ra[j] = make_uint4(0, 0, 0, 0);
    }
  };
  auto fetch_b = [&](int chunk, int grp, uint4 (&r)[BV]) {      // filter row `grp` (= kd * 3 + kh) of a channel block
    const uint16_t* bt = p.B + grp * b_group_stride + chunk * BK;
#pragma unroll
    for (int j = 0; j < BV; ++j) {
      const int c = chunk * BK + ((tid + j * NTHREADS) & 3) * 8;
      if (chunk < nchunks && b_ok[j] && c < p.red) r[j] = *reinterpret_cast<const uint4*>(bt + b_off[j]);
      else r[j] = make_uint4(0, 0, 0, 0);
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
#pragma unroll
  for (int u = 0; u < RBD; ++u) fetch_b(0, u, rb[u]);

  const bool vec_ok = (p.nout & 7) == 0;

  int buf = 0;
  for (int chunk = 0; chunk < nchunks; ++chunk) {
    __syncthreads();                       // every wave is done reading the previous channel block
#pragma unroll
    for (int j = 0; j < AV; ++j) {
      const int v = tid + j * NTHREADS;
      if ((v >> 2) < PT::MAXPIX) *reinterpret_cast<uint4*>(sA + ((v >> 2) / PT::HW) * ROWP + ((v >> 2) % PT::HW) * LDA + (v & 3) * 8) = ra[j];
    }
    if (chunk + 1 < nchunks) fetch_a(chunk + 1);
    for (int kd = 0; kd < KD; ++kd) {
#pragma unroll
      for (int u = 0; u < 3; ++u) {          // filter row kh = u of plane kd
        uint4 (&rcur)[BV] = rb[RBD == 3 ? u : 0];
        uint16_t* b = sB + buf * B_ELEMS;
#pragma unroll
        for (int j = 0; j < BV; ++j) {
          const int v = tid + j * NTHREADS;
          if ((v >> 2) < G_TAPS * BN) *reinterpret_cast<uint4*>(b + (v >> 2) * LDA + (v & 3) * 8) = rcur[j];
        }
        __syncthreads();
        {   // RBD stages ahead: a later row of this channel block or a row of the next one
          int fg = kd * 3 + u + RBD, fc = chunk;
          if (fg >= 3 * KD) { fg -= 3 * KD; ++fc; }
          fetch_b(fc, fg, rcur);
        }
        const int jd = FLIP ? KD - 1 - kd : kd;
        const int jh = FLIP ? 2 - u : u;
        const int row_off = (jd * PT::HH + jh) * ROWP;
        const uint16_t* a_row[TM];
        const uint16_t* b_row[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a_row[i] = sA + a_pix[i] + row_off + (lane >> 5) * 8;
#pragma unroll
        for (int j = 0; j < TN; ++j) b_row[j] = b + (wn * WTN + j * 32 + (lane & 31)) * LDA + (lane >> 5) * 8;
        // six steps (3 taps x 2 halves of the channel block); with PIPE the operands of step s+1 are read from LDS
        // while the products of step s run: two fragment sets, the interleaving is pinned for the scheduler below
        constexpr int NSTEP = G_TAPS * (BK / 16);
        bf16x8 af[PIPE ? 2 : 1][TM], bfr[PIPE ? 2 : 1][TN];
        auto load_step = [&](int st, int slot) {
          const int tl = st / (BK / 16), ks = st % (BK / 16);
          const int jw = FLIP ? G_TAPS - 1 - tl : tl;
#pragma unroll
          for (int i = 0; i < TM; ++i) af[slot][i] = *reinterpret_cast<const bf16x8*>(a_row[i] + jw * LDA + ks * 16);
#pragma unroll
          for (int j = 0; j < TN; ++j) bfr[slot][j] = *reinterpret_cast<const bf16x8*>(b_row[j] + tl * BN * LDA + ks * 16);
        };
        if (PIPE) load_step(0, 0);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
          if (!PIPE) load_step(st, 0);
          else if (st + 1 < NSTEP) load_step(st + 1, (st + 1) & 1);
          constexpr int one = PIPE ? 1 : 0;
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[st & one][j], af[st & one][i], acc[i][j], 0, 0, 0);
        }
        if (PIPE) {
          __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);             // LDS reads of step 0
#pragma unroll
          for (int st = 0; st + 1 < NSTEP; ++st) {
            __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);           // reads of step st+1
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);           // products of step st
          }
          __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
        }
        buf ^= 1;
      }
    }
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

template <int P3D, int BM, int BN, int WM, int WN, int FLIP>
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
  const long long nt = batch * hp.tiles[0] * hp.tiles[1] * hp.tiles[2] * hp.ntiles_n;
  if (nt > 0x7fffff00LL) return hipErrorInvalidValue;
  hp.ntiles = (int)nt;
  const int grid = 8 * ((hp.ntiles + 7) / 8);
  hipLaunchKernelGGL((conv_halo_kernel<P3D, BM, BN, WM, WN, FLIP>), dim3(grid), dim3(NTHREADS), 0, s, hp);
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
