// Resident-filter convolution for the two small-channel 3x3 shapes that dominate the largest feature maps:
// 2-D 3x3 with 64 -> 64 channels and 3-D 3x3x3 with 32 -> 32 channels, stride 1 (forward and data gradient).
//
// The whole filter (72 KB / 54 KB in bf16) is small enough to live in the registers of a work-group as MFMA
// operand fragments: each of the four waves keeps all taps for all output channels (288 / 216 registers per
// lane).  One work-group per compute unit is launched and walks over output patches (2-D: 8x16, 3-D: 4x8x8
// positions).  Per patch the only LDS traffic is the input patch with its halo, all channels at once: it is
// fetched from global memory into registers while the previous patch is multiplied, written to the other half
// of a double buffer, and one barrier per patch separates the two.  The filter is never re-read and there is
// no barrier inside the reduction over taps and channels.
//
// A wave issues its vector instructions and its matrix instructions one after the other (with one wave per SIMD
// nothing else fills the gaps), so everything besides the products is kept short: the filter fragments sit in the
// accumulation registers and are named directly as operands of the matrix instruction (written as inline assembly
// for that reason: the compiler would copy them to ordinary registers first), global memory is reached through
// buffer descriptors so that padding needs no branches, and the stores of a patch are issued one patch late so
// that no wait for loads ever covers a fresh store.
//
// Products are taken transposed (filter fragment as first operand) so that a lane ends up with consecutive
// output channels of one position and stores 16-byte vectors directly from the accumulators.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

template <int P3D>
struct RfShape {
  static constexpr int C = P3D ? 32 : 64;            // input (reduction) channels
  static constexpr int K = P3D ? 32 : 64;            // output channels
  static constexpr int TD = P3D ? 4 : 1, TH = 8, TW = P3D ? 8 : 16;      // output patch
  static constexpr int TM = P3D ? 2 : 1;             // 32-position MFMA tiles per wave
  static constexpr int TN = K / 32;
  static constexpr int KS = C / 16;                  // reduction steps per tap
  static constexpr int KD = P3D ? 3 : 1;
  static constexpr int TAPS = KD * 9;
  static constexpr int BM = TD * TH * TW;            // = 4 waves x TM x 32
  static constexpr int HD = TD + KD - 1, HH = TH + 2, HW = TW + 2;
  static constexpr int NPIX = HD * HH * HW;
  static constexpr int PITCH = C + 8;                // LDS pixel pitch (bf16): 144 / 80 bytes, conflict-free 16-byte reads
  static constexpr int VPP = C / 8;                  // 16-byte vectors per pixel
  static constexpr int NVEC = NPIX * VPP;
  static constexpr int AV = (NVEC + NTHREADS - 1) / NTHREADS;
  // A 16-byte read covers 16 lanes per cycle.  With 16 positions per patch row (2-D) these are one halo row at pixel
  // pitch: conflict-free.  With 8 per row (3-D) they are two halo rows, whose bank sets are disjoint only if the rows
  // lie 128 bytes apart modulo 256: 10 pixels of 80 bytes are 32 modulo 256, hence 96 bytes of padding per row.
  static constexpr int ROWP = HW * PITCH + (P3D ? 48 : 0);            // LDS halo row pitch (bf16)
  static constexpr int BUF = HD * HH * ROWP + 8;     // elements per LDS buffer; the last 16 bytes take the writes of idle lanes
  static constexpr int WROWS = TAPS * K;             // filter rows of C channels, staged through LDS once at the start
  static constexpr int WVEC = WROWS * VPP;
  static constexpr int NFRAG = TAPS * KS * TN;       // filter fragments per lane (4 registers each)
  static constexpr int NFRAG_A = NFRAG < 64 ? NFRAG : 64;   // the first 64 live in the 256 accumulation registers
  static constexpr int LBT = K == 64 ? 96 : 32;      // pitch of the filter as stored, [tap][c][k] rows of K: 64 bytes modulo 256
  static constexpr int WSTAGE = WROWS * PITCH > TAPS * C * LBT ? WROWS * PITCH : TAPS * C * LBT;
  static constexpr int LDS_BYTES = (2 * BUF > WSTAGE ? 2 * BUF : WSTAGE) * 2;
};

// stand-ins for an absent per-channel scale / shift, so that the epilogue needs no branch
__device__ const float rf_ones[64] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f,
                                       1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f,
                                       1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
__device__ const float rf_zeros[64] = {};

#ifndef RF_PD
#define RF_PD 4
#endif
struct RfP {
  IgemmP g;
  int org[3];              // source coordinate of halo index 0 relative to the patch origin
  int tiles[3];            // patches per axis
  int ntiles;
  int per_xcd;             // patches per XCD (contiguous range)
  int wgs_per_xcd;
  int step[4];             // wgs_per_xcd decomposed over (batch, tiles[0], tiles[1], tiles[2])
  unsigned a_bytes, o_bytes;   // sizes of the input and output tensors (below 2 GiB: offsets are 32-bit)
};

typedef int v4i __attribute__((ext_vector_type(4)));

// acc (+)= w * x with the filter fragment w in accumulation registers (ACC) or ordinary ones; FIRST: acc = w * x.
template <bool ACC, bool FIRST>
__device__ __forceinline__ void rf_mfma(f32x16& acc, const v4i& w, const v4i& x) {
  if (FIRST) {
    if (ACC) asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "a"(w), "v"(x));
    else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(w), "v"(x));
  } else {
    if (ACC) asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "a"(w), "v"(x));
    else asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(w), "v"(x));
  }
}

// EPI: which epilogue terms the launch has (bit 0: tensor added, bit 1: ReLU mask tensor, bit 2: per-channel scale or
// shift).  They are template parameters so that the epilogue is straight-line code: all loads before the products,
// all stores together at the end of a patch, no branch in between that would make a wait cover the stores.
template <int P3D, int FLIP, int EPI>
__global__ __launch_bounds__(NTHREADS, 1) void conv_rf_kernel(RfP rp) {
  typedef RfShape<P3D> S;
  extern __shared__ __attribute__((aligned(16))) unsigned char rf_smem[];
  uint16_t* sA = reinterpret_cast<uint16_t*>(rf_smem);
  const IgemmP& p = rp.g;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- patches of this work-group: xcd * per_xcd + slot, then every wgs_per_xcd-th one of the XCD's range ----
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  int tile = xcd * rp.per_xcd + slot;
  const int tile_end = min((xcd + 1) * rp.per_xcd, rp.ntiles);
  if (tile >= tile_end) return;
  int tw, th, td, nb;
  {
    int t = tile;
    tw = t % rp.tiles[2]; t /= rp.tiles[2];
    th = t % rp.tiles[1]; t /= rp.tiles[1];
    td = t % rp.tiles[0]; t /= rp.tiles[0];
    nb = t;
  }

  // Global memory is reached through buffer descriptors with 32-bit byte offsets: an offset at or beyond the
  // tensor size reads zeros and drops writes, so padding, ragged patches and idle lanes need no branch.
  constexpr int OOB = (int)0x80000000;
  constexpr int RSRC = 0x00020000;
  const __amdgpu_buffer_rsrc_t rs_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.A), 0, (int)rp.a_bytes, RSRC);
  const __amdgpu_buffer_rsrc_t rs_o = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, (int)rp.o_bytes, RSRC);
  const __amdgpu_buffer_rsrc_t rs_add = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.add), 0, (EPI & 1) ? (int)rp.o_bytes : 0, RSRC);
  const __amdgpu_buffer_rsrc_t rs_mask = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.mask), 0, (EPI & 2) ? (int)rp.o_bytes : 0, RSRC);

  // ---- halo vectors of this thread (the same for every patch): byte offset from the halo origin, LDS slot, halo index ----
  int a_rel[S::AV], a_lds[S::AV], a_idx[S::AV];
#pragma unroll
  for (int j = 0; j < S::AV; ++j) {
    const int v = tid + j * NTHREADS;
    const int pix = v / S::VPP, cv = v % S::VPP;
    const int jw = pix % S::HW, jh = (pix / S::HW) % S::HH, jd = pix / (S::HW * S::HH);
    const bool used = v < S::NVEC;
    a_rel[j] = (((jd * p.asp[1] + jh) * p.asp[2] + jw) * S::C + cv * 8) * 2;
    a_lds[j] = used ? (jd * S::HH + jh) * S::ROWP + jw * S::PITCH + cv * 8 : S::BUF - 8;
    a_idx[j] = used ? (jd << 20) | (jh << 10) | jw : 0x3fffffff;       // idle lanes: beyond every feature map
  }
  // ---- per-lane constants of the MFMA tiles: halo pixel of the first tap, patch-local output position and offset ----
  int a_frag[S::TM], o_loc[S::TM], o_rel[S::TM];
#pragma unroll
  for (int i = 0; i < S::TM; ++i) {
    const int m = (wave * S::TM + i) * 32 + (lane & 31);
    const int pw = m % S::TW, ph = (m / S::TW) % S::TH, pd = m / (S::TW * S::TH);
    a_frag[i] = (pd * S::HH + ph) * S::ROWP + pw * S::PITCH + (lane >> 5) * 8;
    o_loc[i] = (pd << 20) | (ph << 10) | pw;
    o_rel[i] = ((((pd * p.osp[1] + ph) * p.osp[2] + pw) * S::K) + (lane >> 5) * 8) * 2;
  }

  v4i ra[S::AV];
  auto fetch_a = [&](bool valid, int fnb, int ftd, int fth, int ftw) {
    const int h0d = ftd * S::TD + rp.org[0], h0h = fth * S::TH + rp.org[1], h0w = ftw * S::TW + rp.org[2];
    const int a_base = ((((fnb * p.asp[0] + h0d) * p.asp[1] + h0h) * p.asp[2] + h0w) * S::C) * 2;
#pragma unroll
    for (int j = 0; j < S::AV; ++j) {
      const int id = h0d + (a_idx[j] >> 20), ih = h0h + ((a_idx[j] >> 10) & 1023), iw = h0w + (a_idx[j] & 1023);
      const bool ok = valid && (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] && (unsigned)iw < (unsigned)p.asp[2];
      ra[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_a, ok ? a_base + a_rel[j] : OOB, 0, 0);
    }
  };
  auto store_a = [&](int buf) {
    uint16_t* dst = sA + buf * S::BUF;
#pragma unroll
    for (int j = 0; j < S::AV; ++j) *reinterpret_cast<v4i*>(dst + a_lds[j]) = ra[j];
  };

  fetch_a(true, nb, td, th, tw);        // the first patch is on its way while the filter is set up

  // ---- the filter, resident: copied to LDS with full-width loads, then every lane picks its fragments
  // (tap, step, channel tile) = 8 reduction channels of one output channel.  The data gradient reduces over the
  // last axis of the stored filter [tap][c][k]: rows are read as they lie.  The forward pass reduces over c: the
  // fragments are gathered with the transposing LDS read, so the filter needs no repacking pass. ----
  constexpr int WROW_V = FLIP ? S::VPP : S::K / 8;                   // 16-byte vectors per staged row
  constexpr int WPITCH = FLIP ? S::PITCH : S::LBT;
  {
    constexpr int WV = (S::WVEC + NTHREADS - 1) / NTHREADS;
    v4i wq[WV];
#pragma unroll
    for (int q = 0; q < WV; ++q) {
      const int v = tid + q * NTHREADS;
      if (v < S::WVEC) wq[q] = *reinterpret_cast<const v4i*>(p.B + (long long)v * 8);
    }
#pragma unroll
    for (int q = 0; q < WV; ++q) {
      const int v = tid + q * NTHREADS;
      if (v < S::WVEC) *reinterpret_cast<v4i*>(sA + (v / WROW_V) * WPITCH + (v % WROW_V) * 8) = wq[q];
    }
  }
  __syncthreads();
  v4i wf[S::NFRAG];
  if (FLIP) {
    const uint16_t* wrow = sA + (lane & 31) * S::PITCH + (lane >> 5) * 8;
#pragma unroll
    for (int t = 0; t < S::TAPS; ++t)
#pragma unroll
      for (int ks = 0; ks < S::KS; ++ks)
#pragma unroll
        for (int j = 0; j < S::TN; ++j)
          wf[(t * S::KS + ks) * S::TN + j] = *reinterpret_cast<const v4i*>(wrow + (t * S::K + j * 32) * S::PITCH + ks * 16);
  } else {
    typedef short v4s __attribute__((ext_vector_type(4)));
    typedef short v8s __attribute__((ext_vector_type(8)));
    const int lg = lane >> 4, li = lane & 15;
    const uint16_t* wq0 = sA + (8 * (lg >> 1) + (li >> 2)) * S::LBT + 16 * (lg & 1) + 4 * (li & 3);
#pragma unroll
    for (int t = 0; t < S::TAPS; ++t)
#pragma unroll
      for (int ks = 0; ks < S::KS; ++ks)
#pragma unroll
        for (int j = 0; j < S::TN; ++j) {
          const uint16_t* q = wq0 + (t * S::C + ks * 16) * S::LBT + 32 * j;
          const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)q);
          const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(q + 4 * S::LBT));
          const v8s r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          wf[(t * S::KS + ks) * S::TN + j] = __builtin_bit_cast(v4i, r);
        }
  }
  __syncthreads();                      // the staging area is the first patch buffer
  store_a(0);
  __syncthreads();

  // The stores of a patch are issued one patch late, after the loads of the following iteration: every wait for
  // loads then finds the older stores long finished instead of stalling on them.
  v4i outq[S::TM][S::TN][2];
  int s_off[S::TM];
#pragma unroll
  for (int i = 0; i < S::TM; ++i) s_off[i] = OOB;
  auto store_out = [&]() {
#pragma unroll
    for (int i = 0; i < S::TM; ++i)
#pragma unroll
      for (int j = 0; j < S::TN; ++j)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) __builtin_amdgcn_raw_buffer_store_b128(outq[i][j][pr], rs_o, s_off[i] + (j * 32 + pr * 16) * 2, 0, 0);
  };

  int buf = 0;
  for (;;) {
    __builtin_amdgcn_s_waitcnt(0x0f70);       // vmcnt(0): nothing recent is in flight here
    // next patch of this work-group: coordinates advance by wgs_per_xcd in mixed radix
    const int ntile = tile + rp.wgs_per_xcd;
    const bool more = ntile < tile_end;
    int ntw = tw + rp.step[3], nth = th, ntd = td, nnb = nb;
    {
      int c = ntw >= rp.tiles[2]; ntw -= c ? rp.tiles[2] : 0;
      nth += rp.step[2] + c; c = nth >= rp.tiles[1]; nth -= c ? rp.tiles[1] : 0;
      ntd += rp.step[1] + c; c = ntd >= rp.tiles[0]; ntd -= c ? rp.tiles[0] : 0;
      nnb += rp.step[0] + c;
    }
    fetch_a(more, nnb, ntd, nth, ntw);                 // in flight while this patch is multiplied (nothing after the last one)

    // ---- output offsets of this patch and the tensors the epilogue adds / masks with, fetched early ----
    int o_off[S::TM];
    const int o_base = ((((nb * p.osp[0] + td * S::TD) * p.osp[1] + th * S::TH) * p.osp[2] + tw * S::TW) * S::K) * 2;
#pragma unroll
    for (int i = 0; i < S::TM; ++i) {
      const int od = td * S::TD + (o_loc[i] >> 20), oh = th * S::TH + ((o_loc[i] >> 10) & 1023), ow = tw * S::TW + (o_loc[i] & 1023);
      const bool ok = od < p.osp[0] && oh < p.osp[1] && ow < p.osp[2];
      o_off[i] = ok ? o_base + o_rel[i] : OOB;
    }
    v4i addq[S::TM][S::TN][2], maskq[S::TM][S::TN][2];
#pragma unroll
    for (int i = 0; i < S::TM; ++i)
#pragma unroll
      for (int j = 0; j < S::TN; ++j)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          if (EPI & 1) addq[i][j][pr] = __builtin_amdgcn_raw_buffer_load_b128(rs_add, o_off[i] + (j * 32 + pr * 16) * 2, 0, 0);
          if (EPI & 2) maskq[i][j][pr] = __builtin_amdgcn_raw_buffer_load_b128(rs_mask, o_off[i] + (j * 32 + pr * 16) * 2, 0, 0);
        }

    store_out();                                       // the previous patch (nothing in the first iteration)

    // ---- all taps and channels of this patch: one LDS read per 32 positions and step, filter from registers.
    // The operands of step s+PD are read from LDS while the products of step s run: a ring of PD+1 fragment sets. ----
    f32x16 acc[S::TM][S::TN];
    const uint16_t* a_cur = sA + buf * S::BUF;
    constexpr int NSTEP = S::TAPS * S::KS;
    constexpr int PD = RF_PD;
    v4i af[PD + 1][S::TM];
    auto load_step = [&](int st, int slot) {
      const int t = st / S::KS, ks = st % S::KS;
      const int kw = t % 3, kh = (t / 3) % 3, kd = t / 9;
      const int jw = FLIP ? 2 - kw : kw, jh = FLIP ? 2 - kh : kh, jd = FLIP ? S::KD - 1 - kd : kd;
      const int tap_off = (jd * S::HH + jh) * S::ROWP + jw * S::PITCH;
#pragma unroll
      for (int i = 0; i < S::TM; ++i) af[slot][i] = *reinterpret_cast<const v4i*>(a_cur + a_frag[i] + tap_off + ks * 16);
    };
#pragma unroll
    for (int st = 0; st < PD; ++st) load_step(st, st);
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
      if (st + PD < NSTEP) load_step(st + PD, (st + PD) % (PD + 1));
#pragma unroll
      for (int i = 0; i < S::TM; ++i)
#pragma unroll
        for (int j = 0; j < S::TN; ++j) {
          constexpr int dummy = 0; (void)dummy;
          const int f = st * S::TN + j;
          if (st == 0) {
            if (f < S::NFRAG_A) rf_mfma<true, true>(acc[i][j], wf[f], af[st % (PD + 1)][i]);
            else rf_mfma<false, true>(acc[i][j], wf[f], af[st % (PD + 1)][i]);
          } else {
            if (f < S::NFRAG_A) rf_mfma<true, false>(acc[i][j], wf[f], af[st % (PD + 1)][i]);
            else rf_mfma<false, false>(acc[i][j], wf[f], af[st % (PD + 1)][i]);
          }
        }
      __builtin_amdgcn_sched_barrier(0);        // keep the reads PD steps ahead of their use, no further
    }
    // The compiler does not know these are matrix instructions and inserts no wait states for them: results may be
    // read 18 wait states after the last one at the earliest.  The wait takes both accumulators as in/out operands,
    // so it cannot move above the last product nor any read of a result above it, whatever the scheduler does.
    // (Operands: the filter fragments are written once before the patch loop, the input fragments come from LDS reads
    // that the compiler waits for because the asm statements name their registers.)
    static_assert(S::TM * S::TN == 2, "the wait below names the two accumulator tiles");
    asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc[0][0]), "+v"(acc[S::TM - 1][S::TN - 1]) : : "memory");

    // ---- epilogue: a lane holds 16 channels of one position per tile, 4 consecutive ones per register group with
    // the half-waves interleaved; one cross-half swap per register pair leaves 8 consecutive channels per lane ----
    const float* scp = p.scale ? p.scale : rf_ones;
    const float* shp = p.shift ? p.shift : rf_zeros;
    const bool relu = p.relu != 0;
#pragma unroll
    for (int i = 0; i < S::TM; ++i)
#pragma unroll
      for (int j = 0; j < S::TN; ++j)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          float x[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[i][j][8 * pr + e]),
                                                             __float_as_uint(acc[i][j][8 * pr + 4 + e]), false, false);
            x[e] = __uint_as_float(sw[0]);
            x[4 + e] = __uint_as_float(sw[1]);
          }
          const int n = j * 32 + pr * 16 + (lane >> 5) * 8;
          if (EPI & 4) {
            const float4 s0 = *reinterpret_cast<const float4*>(scp + n), s1 = *reinterpret_cast<const float4*>(scp + n + 4);
            const float4 h0 = *reinterpret_cast<const float4*>(shp + n), h1 = *reinterpret_cast<const float4*>(shp + n + 4);
            const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            const float sh[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(x[e], sc[e], sh[e]);
          }
          if (EPI & 1) {
            const uint32_t aw[4] = {(uint32_t)addq[i][j][pr].x, (uint32_t)addq[i][j][pr].y, (uint32_t)addq[i][j][pr].z, (uint32_t)addq[i][j][pr].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] += __uint_as_float((e & 1) ? (aw[e >> 1] & 0xffff0000u) : (aw[e >> 1] << 16));
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float r = __builtin_amdgcn_fmed3f(x[e], 0.f, __builtin_inff());      // NaN -> 0 like fmaxf
            x[e] = relu ? r : x[e];
          }
          if (EPI & 2) {
            const uint32_t mw[4] = {(uint32_t)maskq[i][j][pr].x, (uint32_t)maskq[i][j][pr].y, (uint32_t)maskq[i][j][pr].z, (uint32_t)maskq[i][j][pr].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float mv = __uint_as_float((e & 1) ? (mw[e >> 1] & 0xffff0000u) : (mw[e >> 1] << 16));
              x[e] = mv > 0.f ? x[e] : 0.f;
            }
          }
          outq[i][j][pr] = v4i{(int)pack_bf16x2(x[0], x[1]), (int)pack_bf16x2(x[2], x[3]), (int)pack_bf16x2(x[4], x[5]), (int)pack_bf16x2(x[6], x[7])};
        }
#pragma unroll
    for (int i = 0; i < S::TM; ++i) s_off[i] = o_off[i];
    if (!more) break;
    store_a(buf ^ 1);
    __syncthreads();            // the next patch is in LDS; every wave is done reading this one
    buf ^= 1;
    tile = ntile; tw = ntw; th = nth; td = ntd; nb = nnb;
  }
  store_out();
}

template <int P3D, int FLIP, int EPI>
hipError_t launch_rf_e(const RfP& rp, int grid, hipStream_t s) {
  typedef RfShape<P3D> S;
  static bool attr_set = false;      // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_rf_kernel<P3D, FLIP, EPI>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((conv_rf_kernel<P3D, FLIP, EPI>), dim3(grid), dim3(NTHREADS), S::LDS_BYTES, s, rp);
  return hipGetLastError();
}

template <int P3D, int FLIP>
hipError_t launch_rf_t(RfP& rp, int cus, hipStream_t s) {
  const int grid = 8 * (cus / 8);
  rp.wgs_per_xcd = grid / 8;
  rp.per_xcd = (rp.ntiles + 7) / 8;
  int rest = rp.wgs_per_xcd;
  rp.step[3] = rest % rp.tiles[2]; rest /= rp.tiles[2];
  rp.step[2] = rest % rp.tiles[1]; rest /= rp.tiles[1];
  rp.step[1] = rest % rp.tiles[0]; rest /= rp.tiles[0];
  rp.step[0] = rest;
  const IgemmP& p = rp.g;
  const int epi = (p.add ? 1 : 0) | (p.mask ? 2 : 0) | ((p.scale || p.shift) ? 4 : 0);
  switch (epi) {
    case 0: return launch_rf_e<P3D, FLIP, 0>(rp, grid, s);
    case 1: return launch_rf_e<P3D, FLIP, 1>(rp, grid, s);
    case 2: return launch_rf_e<P3D, FLIP, 2>(rp, grid, s);
    case 3: return launch_rf_e<P3D, FLIP, 3>(rp, grid, s);
    case 4: return launch_rf_e<P3D, FLIP, 4>(rp, grid, s);
    case 5: return launch_rf_e<P3D, FLIP, 5>(rp, grid, s);
    case 6: return launch_rf_e<P3D, FLIP, 6>(rp, grid, s);
    default: return launch_rf_e<P3D, FLIP, 7>(rp, grid, s);
  }
}

int rf_compute_units() {
  static int cus = -1;
  if (cus < 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    cus = n;
  }
  return cus;
}

template <int P3D>
long long rf_tiles(const IgemmP& p, int* tiles) {
  typedef RfShape<P3D> S;
  tiles[0] = (p.osp[0] + S::TD - 1) / S::TD;
  tiles[1] = (p.osp[1] + S::TH - 1) / S::TH;
  tiles[2] = (p.osp[2] + S::TW - 1) / S::TW;
  const long long batch = p.M / ((long long)p.osp[0] * p.osp[1] * p.osp[2]);
  return batch * tiles[0] * tiles[1] * tiles[2];
}

}  // namespace

bool rf_eligible(const IgemmP& p) {
  static const bool off = getenv("LMS_NO_RF") != nullptr;      // tuning aid: leave these shapes to the patch-tiled kernel
  if (off || p.small || (p.mode != 0 && p.mode != 1)) return false;
  const bool p3d = p.filt[0] == 3;
  if (p.filt[1] != 3 || p.filt[2] != 3 || (p.filt[0] != 1 && p.filt[0] != 3)) return false;
  for (int i = 0; i < 3; ++i)
    if (p.stride[i] != 1) return false;
  if (p3d ? (p.red != 32 || p.nout != 32) : (p.red != 64 || p.nout != 64)) return false;
  if (p.asp[0] >= 1000 || p.asp[1] >= 1000 || p.asp[2] >= 1000) return false;   // halo indices are packed in 10 bits
  const long long batch = p.M / ((long long)p.osp[0] * p.osp[1] * p.osp[2]);
  const long long a_bytes = batch * p.asp[0] * p.asp[1] * p.asp[2] * p.red * 2, o_bytes = p.M * p.nout * 2;
  if (a_bytes >= 0x7fffff00LL || o_bytes >= 0x7fffff00LL) return false;             // 32-bit buffer offsets
  const int cus = rf_compute_units();
  if (cus < 8) return false;
  int tiles[3];
  const long long nt = p3d ? rf_tiles<1>(p, tiles) : rf_tiles<0>(p, tiles);
  // a work-group loads the whole filter once: worth it from a few patches per compute unit on
  return nt >= 3LL * cus && nt < 0x7fffff00LL;
}

hipError_t launch_rf(IgemmP& p, hipStream_t s) {
  RfP rp{};
  rp.g = p;
  for (int i = 0; i < 3; ++i) rp.org[i] = p.mode == 0 ? -p.pad[i] : p.pad[i] - (p.filt[i] - 1);
  const bool p3d = p.filt[0] == 3;
  rp.ntiles = (int)(p3d ? rf_tiles<1>(p, rp.tiles) : rf_tiles<0>(p, rp.tiles));
  const long long batch = p.M / ((long long)p.osp[0] * p.osp[1] * p.osp[2]);
  rp.a_bytes = (unsigned)(batch * p.asp[0] * p.asp[1] * p.asp[2] * p.red * 2);
  rp.o_bytes = (unsigned)(p.M * p.nout * 2);
  const int cus = rf_compute_units();
  if (p.mode == 1) return p3d ? launch_rf_t<1, 1>(rp, cus, s) : launch_rf_t<0, 1>(rp, cus, s);
  return p3d ? launch_rf_t<1, 0>(rp, cus, s) : launch_rf_t<0, 0>(rp, cus, s);
}

}  // namespace lms
