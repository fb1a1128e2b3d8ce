// Implicit-GEMM convolution kernels for gfx950 (CDNA4): forward, data gradient, weight gradient,
// 2-D and 3-D, bf16 operands, fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//
// Forward and data gradient share one kernel: out[m][n] = epi(sum_{tap,r} A[src(m,tap)][r] * B[tap][n][r])
// where m runs over output positions (channels-last rows), A rows are gathered per filter tap and B is
// the filter with the reduction index contiguous.  Tiles of A and B are staged through LDS with
// 16-byte loads along the channel axis; the accumulators are transposed through LDS once more so
// that the epilogue (scale/shift, residual or gradient add, ReLU or ReLU mask) reads and writes
// 16-byte channel vectors.
//
// The weight gradient reduces over positions, so both operands have to be transposed on their way
// into the MFMA; this happens while writing the LDS tiles (pairs of positions are packed into
// 32-bit words, rows are XOR-swizzled).  The position range is split over work-groups and the
// partial filters are summed in a fixed order by a second kernel, so results do not depend on
// scheduling.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <type_traits>

#include "kernels.hpp"
#include "conv_common.hpp"

namespace lms {

namespace {

// Source position of output position o for filter tap t along one axis; -1 if outside / not on the lattice.
__device__ __forceinline__ int src_coord(int o, int t, int stride, int pad, int extent, int mode) {
  if (mode == 0) {
    int i = o * stride + t - pad;
    return (i >= 0 && i < extent) ? i : -1;
  }
  int i = o + pad - t;
  if (i < 0) return -1;
  int q = i / stride;
  if (q * stride != i || q >= extent) return -1;
  return q;
}

// Gather modes of the implicit-GEMM kernel (template parameter GM):
//   GM_FWD    src = o*stride + tap - pad            (forward convolution, any stride): linear in the tap
//   GM_TR1    src = o + pad - tap                   (data gradient of a stride-1 convolution): linear
//   GM_TRS    src = (o + pad - tap) / stride        (data gradient with stride > 1, transposed-conv forward)
//   GM_SMALL  (tap, channel) flattened, element-wise gather (channel counts that are not a multiple of 8)
//   GM_TRC    as GM_TRS, with the output positions tiled by residue class: the positions o = stride*q + a of one
//             class a (per axis) see exactly the taps t = (a + pad) mod stride, + stride, ..., and their source is
//             q + (a + pad - t)/stride: linear again.  A tile lies within one class, so it runs over the taps of
//             its class only (a quarter of them for stride 2 in two dimensions) and never fetches a zero row.
//             Needs output extents that are multiples of the strides.
enum { GM_FWD = 0, GM_TR1 = 1, GM_TRS = 2, GM_SMALL = 3, GM_TRC = 4 };

template <int BM, int BN, int WM, int WN, int GM>
__global__ __launch_bounds__(NTHREADS, (BM == 64 ? 4 : 2)) void igemm_kernel(IgemmP p) {
  constexpr int AR = BM / 64;                   // A rows (one 8-element vector each) fetched per thread
  constexpr int WTM = BM / WM, WTN = BN / WN;   // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;   // 32x32 MFMA tiles per wave
  constexpr int LDC = BN + 4;
  constexpr int STAGE = (BM + BN) * LDA;        // bf16 elements per stage
  constexpr int MAIN_BYTES = 2 * STAGE * 2;
  constexpr int EPI_BYTES = BM * LDC * 4;
  constexpr int SMEM = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ unsigned s_orow[GM == GM_TRC ? BM : 1];   // GM_TRC: output row of each tile row
  uint16_t* sA = reinterpret_cast<uint16_t*>(smem);
  float* sC = reinterpret_cast<float*>(smem);

  // Work-groups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so
  // that neighbouring tiles (which share filter taps' halo rows and the filter) share one L2.
  const int per_xcd = (p.ntiles + 7) / 8;
  const int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= p.ntiles) return;
  const int tile_n = tile % p.ntiles_n;
  const int tile_m = tile / p.ntiles_n;
  long long m0 = (long long)tile_m * BM;
  const int n0 = tile_n * BN;
  // GM_TRC: residue class of the tile, its first tap per axis, taps per axis, source shift of the first tap
  int cls_a[3] = {0, 0, 0}, cls_k0[3] = {0, 0, 0}, cls_cnt[3] = {1, 1, 1}, cls_sh[3] = {0, 0, 0};
  if (GM == GM_TRC) {
    // the class is the fastest index: classes differ in their tap counts (some have none), and every XCD should
    // get its share of each; the classes of one row tile also write neighbouring output rows
    const int classes = p.stride[0] * p.stride[1] * p.stride[2];
    int cls = tile_m % classes;
    m0 = (long long)(tile_m / classes) * BM;
    cls_a[2] = cls % p.stride[2]; cls /= p.stride[2];
    cls_a[1] = cls % p.stride[1];
    cls_a[0] = cls / p.stride[1];
#pragma unroll
    for (int d = 0; d < 3; ++d) {
      cls_k0[d] = (cls_a[d] + p.pad[d]) % p.stride[d];
      cls_cnt[d] = cls_k0[d] < p.filt[d] ? (p.filt[d] - cls_k0[d] + p.stride[d] - 1) / p.stride[d] : 0;
      cls_sh[d] = (cls_a[d] + p.pad[d] - cls_k0[d]) / p.stride[d];
    }
  }
  const long long m_lim = (GM == GM_TRC) ? p.Mc : p.M;
  const int* dsp = (GM == GM_TRC) ? p.qsp : p.osp;      // extents the tile rows are decoded with

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- per-thread A rows: AR rows, one 8-element vector each ------------------------------------
  const int avec = tid & 3;
  int a_n[AR], a_o[AR][3];      // batch index; GM_FWD / GM_TR1: first source coordinate, else output coordinate
  long long a_base[AR];         // GM_FWD / GM_TR1: element offset of (n, a_o) (may lie outside the tensor)
  bool a_in[AR];
#pragma unroll
  for (int r = 0; r < AR; ++r) {
    const long long m = m0 + (tid >> 2) + r * 64;
    a_in[r] = m < m_lim;
    unsigned t = a_in[r] ? (unsigned)m : 0u;       // host guarantees M < 2^31
    const unsigned ow = t % (unsigned)dsp[2]; t /= (unsigned)dsp[2];
    const unsigned oh = t % (unsigned)dsp[1]; t /= (unsigned)dsp[1];
    const unsigned od = t % (unsigned)dsp[0]; t /= (unsigned)dsp[0];
    a_n[r] = (int)t;
    if (GM == GM_FWD) {
      a_o[r][0] = (int)od * p.stride[0] - p.pad[0];
      a_o[r][1] = (int)oh * p.stride[1] - p.pad[1];
      a_o[r][2] = (int)ow * p.stride[2] - p.pad[2];
    } else if (GM == GM_TR1) {
      a_o[r][0] = (int)od + p.pad[0];
      a_o[r][1] = (int)oh + p.pad[1];
      a_o[r][2] = (int)ow + p.pad[2];
    } else if (GM == GM_TRC) {
      a_o[r][0] = (int)od + cls_sh[0];
      a_o[r][1] = (int)oh + cls_sh[1];
      a_o[r][2] = (int)ow + cls_sh[2];
      const unsigned o0 = od * p.stride[0] + cls_a[0], o1 = oh * p.stride[1] + cls_a[1], o2 = ow * p.stride[2] + cls_a[2];
      if (avec == 0) s_orow[(tid >> 2) + r * 64] = ((t * p.osp[0] + o0) * p.osp[1] + o1) * p.osp[2] + o2;
    } else {
      a_o[r][0] = (int)od; a_o[r][1] = (int)oh; a_o[r][2] = (int)ow;
    }
    a_base[r] = ((((long long)a_n[r] * p.asp[0] + a_o[r][0]) * p.asp[1] + a_o[r][1]) * p.asp[2] + a_o[r][2]) * p.red;
  }
  // B rows handled by this thread: BN*4 vectors over 256 threads
  constexpr int BV = (BN * 4 + NTHREADS - 1) / NTHREADS;
  long long b_off[BV];
  bool b_ok[BV];
#pragma unroll
  for (int v = 0; v < BV; ++v) {
    const int idx = tid + v * NTHREADS;
    const int row = idx >> 2, cv = (idx & 3) * 8;
    b_ok[v] = row < BN && n0 + row < p.nout;
    b_off[v] = (GM == GM_SMALL) ? (long long)(n0 + row) * p.jpad + cv : (long long)(n0 + row) * p.red + cv;
  }

  if (GM == GM_TRC) __syncthreads();               // s_orow is read before the main loop
  const int chunks_per_tap = (p.red + BK - 1) / BK;
  const int ntap = (GM == GM_TRC) ? cls_cnt[0] * cls_cnt[1] * cls_cnt[2] : p.taps;   // taps this tile runs over
  const int nkh = (GM == GM_TRC) ? cls_cnt[1] : p.filt[1], nkw = (GM == GM_TRC) ? cls_cnt[2] : p.filt[2];
  const int niter = (GM == GM_SMALL) ? p.jpad / BK : ntap * chunks_per_tap;
  const long long b_tap_stride = (long long)p.nout * p.red;

  uint4 ra[2][AR], rb[2][BV];    // two register sets: stages are fetched two iterations ahead
  // state of the next stage to fetch
  int ld_tap = 0, ld_chunk = 0, ld_kd = 0, ld_kh = 0, ld_kw = 0;
  long long pix[AR];             // element offset of the gathered pixel for tap ld_tap, -1 if it is padding
  auto locate_tap = [&]() {
#pragma unroll
    for (int r = 0; r < AR; ++r) {
      if (GM == GM_FWD || GM == GM_TR1 || GM == GM_TRC) {       // GM_TRC: ld_kd, ld_kh, ld_kw count the taps of the class
        const int sg = (GM == GM_FWD) ? 1 : -1;
        const int id = a_o[r][0] + sg * ld_kd, ih = a_o[r][1] + sg * ld_kh, iw = a_o[r][2] + sg * ld_kw;
        const bool ok = a_in[r] && (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] &&
                        (unsigned)iw < (unsigned)p.asp[2];
        const long long toff = ((long long)(ld_kd * p.asp[1] + ld_kh) * p.asp[2] + ld_kw) * p.red;
        pix[r] = ok ? a_base[r] + sg * toff : -1;
      } else {
        const int id = src_coord(a_o[r][0], ld_kd, p.stride[0], p.pad[0], p.asp[0], 1);
        const int ih = src_coord(a_o[r][1], ld_kh, p.stride[1], p.pad[1], p.asp[1], 1);
        const int iw = src_coord(a_o[r][2], ld_kw, p.stride[2], p.pad[2], p.asp[2], 1);
        pix[r] = (a_in[r] && id >= 0 && ih >= 0 && iw >= 0)
                     ? ((((long long)a_n[r] * p.asp[0] + id) * p.asp[1] + ih) * p.asp[2] + iw) * p.red
                     : -1;
      }
    }
  };
  if (GM != GM_SMALL && niter > 0) locate_tap();

  auto load_stage = [&](auto set_c) {
    constexpr int S = decltype(set_c)::value;
    if (GM != GM_SMALL) {
      const int c0 = ld_chunk * BK + avec * 8;
#pragma unroll
      for (int r = 0; r < AR; ++r) {
        if (pix[r] >= 0 && c0 < p.red) ra[S][r] = *reinterpret_cast<const uint4*>(p.A + pix[r] + c0);
        else ra[S][r] = make_uint4(0, 0, 0, 0);
      }
      const int b_tap = (GM == GM_TRC) ? ((cls_k0[0] + p.stride[0] * ld_kd) * p.filt[1] + cls_k0[1] + p.stride[1] * ld_kh) * p.filt[2] +
                                             cls_k0[2] + p.stride[2] * ld_kw
                                       : ld_tap;
      const uint16_t* bt = p.B + b_tap * b_tap_stride + ld_chunk * BK;
#pragma unroll
      for (int v = 0; v < BV; ++v) {
        const int cv = ((tid + v * NTHREADS) & 3) * 8;
        if (b_ok[v] && ld_chunk * BK + cv < p.red) rb[S][v] = *reinterpret_cast<const uint4*>(bt + b_off[v]);
        else rb[S][v] = make_uint4(0, 0, 0, 0);
      }
      if (++ld_chunk == chunks_per_tap) {
        ld_chunk = 0;
        ++ld_tap;
        if (++ld_kw == nkw) {
          ld_kw = 0;
          if (++ld_kh == nkh) { ld_kh = 0; ++ld_kd; }
        }
        if (ld_tap < ntap) locate_tap();
      }
    } else {
      const int j0 = ld_chunk * BK + avec * 8;      // ld_chunk counts stages here
      const int jtot = p.taps * p.red;
#pragma unroll
      for (int r = 0; r < AR; ++r) {
        uint32_t w4[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int j = j0 + i;
          uint32_t val = 0;
          if (a_in[r] && j < jtot) {
            int tap = j / p.red;
            const int c = j - tap * p.red;
            const int kw = tap % p.filt[2]; tap /= p.filt[2];
            const int kh = tap % p.filt[1]; tap /= p.filt[1];
            const int id = src_coord(a_o[r][0], tap, p.stride[0], p.pad[0], p.asp[0], p.mode);
            const int ih = src_coord(a_o[r][1], kh, p.stride[1], p.pad[1], p.asp[1], p.mode);
            const int iw = src_coord(a_o[r][2], kw, p.stride[2], p.pad[2], p.asp[2], p.mode);
            if (id >= 0 && ih >= 0 && iw >= 0)
              val = p.A[((((long long)a_n[r] * p.asp[0] + id) * p.asp[1] + ih) * p.asp[2] + iw) * p.red + c];
          }
          w4[i >> 1] |= val << ((i & 1) * 16);
        }
        ra[S][r] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
      }
#pragma unroll
      for (int v = 0; v < BV; ++v) {
        if (b_ok[v]) rb[S][v] = *reinterpret_cast<const uint4*>(p.B + b_off[v] + ld_chunk * BK);
        else rb[S][v] = make_uint4(0, 0, 0, 0);
      }
      ++ld_chunk;
    }
  };
  auto store_stage = [&](int buf, auto set_c) {
    constexpr int S = decltype(set_c)::value;
    uint16_t* a = sA + buf * STAGE;
    uint16_t* b = a + BM * LDA;
#pragma unroll
    for (int r = 0; r < AR; ++r)
      *reinterpret_cast<uint4*>(a + ((tid >> 2) + r * 64) * LDA + avec * 8) = ra[S][r];
#pragma unroll
    for (int v = 0; v < BV; ++v) {
      const int idx = tid + v * NTHREADS;
      const int row = idx >> 2, cv = (idx & 3) * 8;
      if (row < BN) *reinterpret_cast<uint4*>(b + row * LDA + cv) = rb[S][v];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  typedef std::integral_constant<int, 0> S0;
  typedef std::integral_constant<int, 1> S1;
  if (niter > 0) load_stage(S0{});                 // a class without taps (window smaller than the stride) has none
  if (niter > 1) load_stage(S1{});

  // The epilogue's residual / gradient-add / mask vectors do not depend on the main loop: fetch them
  // now so that their latency hides under it.
  constexpr int EV = BM * (BN / 8) / NTHREADS;
  const bool vec_ok = (p.nout & 7) == 0;
  uint4 pre_add[EV], pre_mask[EV];
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    pre_add[q] = make_uint4(0, 0, 0, 0);
    pre_mask[q] = make_uint4(0, 0, 0, 0);
  }
  if (vec_ok) {
#pragma unroll
    for (int q = 0; q < EV; ++q) {
      const int idx = tid + q * NTHREADS;
      const int r = idx / (BN / 8), cg = (idx % (BN / 8)) * 8;
      const long long m = m0 + r;
      const int n = n0 + cg;
      if (m < m_lim && n < p.nout) {
        const long long orow = (GM == GM_TRC) ? (long long)s_orow[r] : m;
        if (p.add) pre_add[q] = *reinterpret_cast<const uint4*>(p.add + orow * p.nout + n);
        if (p.mask) pre_mask[q] = *reinterpret_cast<const uint4*>(p.mask + orow * p.nout + n);
      }
    }
  }

  if (niter > 0) store_stage(0, S0{});
  __syncthreads();
  auto body = [&](int it, auto set_c) {
    constexpr int S = decltype(set_c)::value;      // == it & 1: LDS buffer and register set of stage `it`
    if (it + 2 < niter) load_stage(set_c);         // stage `it` already sits in LDS: its registers are free
    const uint16_t* a = sA + S * STAGE;
    const uint16_t* b = a + BM * LDA;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
      const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(a + (wm * WTM + i * 32 + (lane & 31)) * LDA + koff);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(b + (wn * WTN + j * 32 + (lane & 31)) * LDA + koff);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (it + 1 < niter) store_stage(S ^ 1, std::integral_constant<int, S ^ 1>{});
    __syncthreads();
  };
  for (int it = 0; it < niter; it += 2) {
    body(it, S0{});
    if (it + 1 < niter) body(it + 1, S1{});
  }

  // ---- epilogue: accumulators -> LDS (row-major fp32) -> 8-channel vectors ---------------------
  // 32x32 accumulator layout: lane l holds column l%32, rows 8*(v/4) + 4*(l/32) + v%4, v = 0..15.
  // A tile of a residue class without taps writes the epilogue of zero and skips the round trip.
  const bool zero_tile = (GM == GM_TRC) && niter == 0;
  if (!zero_tile) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wm * WTM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          const int col = wn * WTN + j * 32 + (lane & 31);
          sC[row * LDC + col] = acc[i][j][v];
        }
    __syncthreads();
  }
  // every vector of this thread has the same channels (the thread count is a multiple of the vectors per row)
  const int cg = (tid % (BN / 8)) * 8, n = n0 + cg;
  const int cnt = (p.nout - n) < 8 ? (p.nout - n) : 8;
  EpiCoef coef;
  if (n < p.nout) epilogue_coef(p, n, cnt, coef);
  uint4 outw[EV];
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    const int r = (tid + q * NTHREADS) / (BN / 8);
    const long long m = m0 + r;
    outw[q] = make_uint4(0, 0, 0, 0);
    if (m >= m_lim || n >= p.nout) continue;
    float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
    if (!zero_tile) {
      lo = *reinterpret_cast<const float4*>(sC + r * LDC + cg);
      hi = *reinterpret_cast<const float4*>(sC + r * LDC + cg + 4);
    }
    const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    const long long off = ((GM == GM_TRC) ? (long long)s_orow[r] : m) * p.nout + n;
    uint4 addq = pre_add[q], maskq = pre_mask[q];
    if (!vec_ok) {
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
    outw[q] = epilogue_pack8(p, coef, v, addq, maskq);
  }
#pragma unroll
  for (int q = 0; q < EV; ++q) {
    const int r = (tid + q * NTHREADS) / (BN / 8);
    const long long m = m0 + r;
    if (m < m_lim && n < p.nout) epilogue_put8(p, outw[q], cnt, ((GM == GM_TRC) ? (long long)s_orow[r] : m) * p.nout + n, vec_ok);
  }
}

// ---------------------------------------------------------------------------------------------
// Weight gradient: part[split][tap][cx][ky] = sum over the split's rows of X[src(m,tap)][cx] * DY[m][ky]
struct WgradP {
  const uint16_t* X;
  const uint16_t* DY;
  float* part;
  long long M;
  int cx, ky;
  int asp[3], osp[3], filt[3], stride[3], pad[3];
  int taps, ctiles, ktiles, splits;
  long long rows_per_split;   // multiple of 64
  int small;                  // cx not a multiple of 8: element-wise loads of X
};

constexpr int WG_T = 64;      // channel tile (both operands) and rows per stage

__device__ __forceinline__ int wg_swz(int c) { return ((c >> 1) & 7) ^ ((c >> 4) & 7); }

__global__ __launch_bounds__(NTHREADS) void wgrad_kernel(WgradP p) {
  // per stage: Xt[64 ch][64 rows] and DYt[64 ch][64 rows] as bf16, rows contiguous, 16-byte units swizzled
  __shared__ __attribute__((aligned(16))) uint32_t smem[2][2][WG_T * 32];
  const int tiles = p.taps * p.ctiles * p.ktiles;
  const int split = blockIdx.x / tiles;
  int tile = blockIdx.x - split * tiles;
  const int kt = tile % p.ktiles; tile /= p.ktiles;
  const int ct = tile % p.ctiles;
  const int tap = tile / p.ctiles;
  const int c0 = ct * WG_T, k0 = kt * WG_T;
  int t = tap;
  const int kw = t % p.filt[2]; t /= p.filt[2];
  const int kh = t % p.filt[1]; t /= p.filt[1];
  const int kd = t;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int pp = tid >> 3;        // row pair 0..31 -> rows 2pp, 2pp+1 of the stage
  const int cv = tid & 7;         // 8-channel vector

  const long long row_begin = (long long)split * p.rows_per_split;
  const long long row_end = (row_begin + p.rows_per_split < p.M) ? row_begin + p.rows_per_split : p.M;
  const int niter = row_end > row_begin ? (int)((row_end - row_begin + WG_T - 1) / WG_T) : 0;

  // Output coordinates of this thread's two rows, advanced by one stage (64 rows) at a time.
  const bool identity = p.taps == 1 && p.stride[0] == 1 && p.stride[1] == 1 && p.stride[2] == 1 &&
                        p.pad[0] == 0 && p.pad[1] == 0 && p.pad[2] == 0;   // 1x1 convolution: source row == output row
  unsigned r_n[2], r_od[2], r_oh[2], r_ow[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    unsigned t = (unsigned)(row_begin + 2 * pp + r);      // host guarantees M < 2^31
    r_ow[r] = t % (unsigned)p.osp[2]; t /= (unsigned)p.osp[2];
    r_oh[r] = t % (unsigned)p.osp[1]; t /= (unsigned)p.osp[1];
    r_od[r] = t % (unsigned)p.osp[0]; t /= (unsigned)p.osp[0];
    r_n[r] = t;
  }
  const bool y_vec = (p.ky & 7) == 0;
  const bool y_in = k0 + cv * 8 < p.ky;
  const bool x_in = c0 + cv * 8 < p.cx;
  long long ld_m = row_begin + 2 * pp;                     // first of the two rows of the next stage to fetch

  uint4 rx[2], ry[2];
  auto load_stage = [&]() {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const long long m = ld_m + r;
      rx[r] = make_uint4(0, 0, 0, 0);
      ry[r] = make_uint4(0, 0, 0, 0);
      if (m < row_end) {
        if (y_in) {
          if (y_vec) ry[r] = *reinterpret_cast<const uint4*>(p.DY + m * p.ky + k0 + cv * 8);
          else {
            uint32_t w4[4] = {0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (k0 + cv * 8 + i < p.ky) w4[i >> 1] |= (uint32_t)p.DY[m * p.ky + k0 + cv * 8 + i] << ((i & 1) * 16);
            ry[r] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
          }
        }
        if (x_in) {
          long long srow = m;
          bool ok = true;
          if (!identity) {
            const int id = (int)r_od[r] * p.stride[0] + kd - p.pad[0];
            const int ih = (int)r_oh[r] * p.stride[1] + kh - p.pad[1];
            const int iw = (int)r_ow[r] * p.stride[2] + kw - p.pad[2];
            ok = (unsigned)id < (unsigned)p.asp[0] && (unsigned)ih < (unsigned)p.asp[1] && (unsigned)iw < (unsigned)p.asp[2];
            srow = (((long long)r_n[r] * p.asp[0] + id) * p.asp[1] + ih) * p.asp[2] + iw;
          }
          if (ok) {
            const uint16_t* src = p.X + srow * p.cx + c0 + cv * 8;
            if (!p.small) rx[r] = *reinterpret_cast<const uint4*>(src);
            else {
              uint32_t w4[4] = {0, 0, 0, 0};
#pragma unroll
              for (int i = 0; i < 8; ++i)
                if (c0 + cv * 8 + i < p.cx) w4[i >> 1] |= (uint32_t)src[i] << ((i & 1) * 16);
              rx[r] = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
          }
        }
      }
      if (!identity) {   // advance this row by one stage
        r_ow[r] += WG_T;
        while (r_ow[r] >= (unsigned)p.osp[2]) {
          r_ow[r] -= (unsigned)p.osp[2];
          if (++r_oh[r] == (unsigned)p.osp[1]) {
            r_oh[r] = 0;
            if (++r_od[r] == (unsigned)p.osp[0]) { r_od[r] = 0; ++r_n[r]; }
          }
        }
      }
    }
    ld_m += WG_T;
  };
  // Transposed store: channel c of rows (2pp, 2pp+1) becomes one 32-bit word of row c of the LDS tile.
  auto store_one = [&](uint32_t* dst, const uint4& r0, const uint4& r1) {
    const uint32_t a[4] = {r0.x, r0.y, r0.z, r0.w};
    const uint32_t b[4] = {r1.x, r1.y, r1.z, r1.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ce = cv * 8 + 2 * i;
      const uint32_t even = (a[i] & 0xffffu) | (b[i] << 16);
      const uint32_t odd = (a[i] >> 16) | (b[i] & 0xffff0000u);
      dst[ce * 32 + (((pp >> 2) ^ wg_swz(ce)) << 2) + (pp & 3)] = even;
      dst[(ce + 1) * 32 + (((pp >> 2) ^ wg_swz(ce + 1)) << 2) + (pp & 3)] = odd;
    }
  };

  f32x16 acc;
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;

  if (niter > 0) {
    load_stage();
    store_one(smem[0][0], rx[0], rx[1]);
    store_one(smem[0][1], ry[0], ry[1]);
  }
  __syncthreads();
  for (int it = 0; it < niter; ++it) {
    const int buf = it & 1;
    if (it + 1 < niter) load_stage();
    const uint32_t* xs = smem[buf][0];
    const uint32_t* ys = smem[buf][1];
    const int rc = wm * 32 + (lane & 31);   // channel row of X tile
    const int rk = wn * 32 + (lane & 31);   // channel row of DY tile
#pragma unroll
    for (int ks = 0; ks < WG_T / 16; ++ks) {
      const int mblk = ks * 2 + (lane >> 5);
      const bf16x8 af = *reinterpret_cast<const bf16x8*>(xs + rc * 32 + ((mblk ^ wg_swz(rc)) << 2));
      const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(ys + rk * 32 + ((mblk ^ wg_swz(rk)) << 2));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc, 0, 0, 0);
    }
    if (it + 1 < niter) {
      store_one(smem[buf ^ 1][0], rx[0], rx[1]);
      store_one(smem[buf ^ 1][1], ry[0], ry[1]);
    }
    __syncthreads();
  }
  float* out = p.part + ((long long)split * p.taps + tap) * p.cx * p.ky;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int c = c0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int k = k0 + wn * 32 + (lane & 31);
    if (c < p.cx && k < p.ky) out[(long long)c * p.ky + k] = acc[v];
  }
}

// dw[idx] = sum_s part[s][idx] in ascending s; optionally written with the last two axes swapped.
__global__ void wgrad_reduce_kernel(const float* part, float* dw, long long per_split, int splits, int taps, int cx,
                                    int ky, int transpose) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= per_split) return;
  float s = 0.f;
  for (int i = 0; i < splits; ++i) s += part[(long long)i * per_split + idx];
  if (!transpose) dw[idx] = s;
  else {
    const int k = (int)(idx % ky);
    const long long r = idx / ky;
    const int c = (int)(r % cx);
    const long long tp = r / cx;
    dw[(tp * ky + k) * cx + c] = s;
  }
}

// Same sum for the common case (no transpose, element count a multiple of 4): every thread adds one eighth
// of the splits for four neighbouring elements, the eight partial sums are then added in a fixed order.
__global__ __launch_bounds__(256) void wgrad_reduce_vec_kernel(const float4* part, float4* dw, long long per4, int splits) {
  __shared__ float4 sh[8][32];
  const int o = threadIdx.x & 31, g = threadIdx.x >> 5;
  const long long idx = (long long)blockIdx.x * 32 + o;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (idx < per4) {
    int i = g;
    for (; i + 24 < splits; i += 32) {
      const float4 a = part[(long long)i * per4 + idx], b = part[(long long)(i + 8) * per4 + idx];
      const float4 c = part[(long long)(i + 16) * per4 + idx], d = part[(long long)(i + 24) * per4 + idx];
      s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
      s.x += b.x; s.y += b.y; s.z += b.z; s.w += b.w;
      s.x += c.x; s.y += c.y; s.z += c.z; s.w += c.w;
      s.x += d.x; s.y += d.y; s.z += d.z; s.w += d.w;
    }
    for (; i < splits; i += 8) {
      const float4 a = part[(long long)i * per4 + idx];
      s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
  }
  sh[g][o] = s;
  __syncthreads();
  if (g == 0 && idx < per4) {
    float4 t = sh[0][o];
#pragma unroll
    for (int j = 1; j < 8; ++j) { t.x += sh[j][o].x; t.y += sh[j][o].y; t.z += sh[j][o].z; t.w += sh[j][o].w; }
    dw[idx] = t;
  }
}

// Filter packing: dst[tap][k][c] = w[tap][c][k] (transpose == 1) or dst = w (transpose == 0), times scale[k].
__global__ void pack_filter_kernel(const uint16_t* w, const float* scale, uint16_t* dst, int taps, int c, int k, int transpose) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)taps * c * k;
  if (idx >= total) return;
  const int kk = (int)(idx % k);
  const long long r = idx / k;
  const int cc = (int)(r % c);
  const long long tp = r / c;
  uint16_t v = w[idx];
  if (scale) v = f2bf(bf2f(v) * scale[kk]);
  if (transpose) dst[(tp * k + kk) * c + cc] = v;
  else dst[idx] = v;
}

// The same for channel counts that are multiples of 8, in 64 x 64 tiles through LDS so that both the reads (k
// contiguous) and the writes (c contiguous after the transposition) are 16-byte vectors.
__global__ __launch_bounds__(256) void pack_filter_tiled_kernel(const uint16_t* w, const float* scale, uint16_t* dst, int c, int k,
                                                                int transpose) {
  __shared__ __attribute__((aligned(16))) uint16_t t[64][72];
  const int k0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const long long tap = blockIdx.z;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int v = threadIdx.x + i * 256;
    const int r = v >> 3, q = (v & 7) * 8;
    uint4 d = make_uint4(0, 0, 0, 0);
    if (c0 + r < c && k0 + q < k) {
      const long long off = (tap * c + c0 + r) * k + k0 + q;
      d = *reinterpret_cast<const uint4*>(w + off);
      if (scale) {
        uint32_t x[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint16_t lo = f2bf(bf2f((uint16_t)(x[e] & 0xffffu)) * scale[k0 + q + 2 * e]);
          const uint16_t hi = f2bf(bf2f((uint16_t)(x[e] >> 16)) * scale[k0 + q + 2 * e + 1]);
          x[e] = (uint32_t)lo | ((uint32_t)hi << 16);
        }
        d = make_uint4(x[0], x[1], x[2], x[3]);
      }
      if (!transpose) *reinterpret_cast<uint4*>(dst + off) = d;
    }
    *reinterpret_cast<uint4*>(&t[r][q]) = d;
  }
  if (!transpose) return;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int v = threadIdx.x + i * 256;
    const int kr = v >> 3, cq = (v & 7) * 8;
    if (k0 + kr < k && c0 + cq < c) {
      uint32_t x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = (uint32_t)t[cq + 2 * e][kr] | ((uint32_t)t[cq + 2 * e + 1][kr] << 16);
      *reinterpret_cast<uint4*>(dst + (tap * k + k0 + kr) * c + c0 + cq) = make_uint4(x[0], x[1], x[2], x[3]);
    }
  }
}

// Launches the packing kernel that fits the channel counts.
static void launch_pack_filter(const uint16_t* w, const float* scale, uint16_t* dst, int taps, int c, int k, int transpose, hipStream_t s) {
  if ((c & 7) == 0 && (k & 7) == 0 && taps < 65536 && (c + 63) / 64 < 65536)
    hipLaunchKernelGGL(pack_filter_tiled_kernel, dim3((k + 63) / 64, (c + 63) / 64, taps), dim3(256), 0, s, w, scale, dst, c, k, transpose);
  else
    hipLaunchKernelGGL(pack_filter_kernel, dim3((unsigned)(((long long)taps * c * k + 255) / 256)), dim3(256), 0, s, w, scale, dst, taps, c, k, transpose);
}

// Small-channel packing: dst[k][tap*c + cc] = w[tap][c][k], rows padded with zeros to jpad.
__global__ void pack_filter_small_kernel(const uint16_t* w, uint16_t* dst, int taps, int c, int k, int jpad) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)k * jpad) return;
  const int j = (int)(idx % jpad);
  const int kk = (int)(idx / jpad);
  dst[idx] = (j < taps * c) ? w[(long long)j * k + kk] : (uint16_t)0;
}

// Same for the data gradient (reduction over output channels k): dst[c][tap*k + kk] = w[tap][c][kk] * scale[kk].
__global__ void pack_filter_small_dgrad_kernel(const uint16_t* w, const float* scale, uint16_t* dst, int taps, int c, int k, int jpad) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)c * jpad) return;
  const int j = (int)(idx % jpad);
  const int cc = (int)(idx / jpad);
  uint16_t v = 0;
  if (j < taps * k) {
    const int tap = j / k, kk = j - tap * k;
    v = w[((long long)tap * c + cc) * k + kk];
    if (scale) v = f2bf(bf2f(v) * scale[kk]);
  }
  dst[idx] = v;
}

inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

void fill_geom(const ConvGeom& g, int* asp, int* osp, int* filt, int* stride, int* pad) {
  for (int i = 0; i < 3; ++i) {
    asp[i] = g.in_sp[i]; osp[i] = g.out_sp[i]; filt[i] = g.filt[i]; stride[i] = g.stride[i]; pad[i] = g.pad[i];
  }
}

template <int BM, int BN, int WM, int WN, int GM>
hipError_t launch_igemm_t(IgemmP& p, hipStream_t s) {
  p.ntiles_n = cdiv(p.nout, BN);
  long long mt = (p.M + BM - 1) / BM;
  if (GM == GM_TRC) {
    const long long classes = (long long)p.stride[0] * p.stride[1] * p.stride[2];
    for (int d = 0; d < 3; ++d) p.qsp[d] = p.osp[d] / p.stride[d];
    p.Mc = p.M / classes;
    const long long ct = (p.Mc + BM - 1) / BM;
    if (ct > 0x7fffff00LL) return hipErrorInvalidValue;
    p.cls_tiles = (int)ct;
    mt = classes * ct;
  }
  if (mt * p.ntiles_n > 0x7fffff00LL || p.M >= 0x7fffffffLL) return hipErrorInvalidValue;
  p.ntiles = (int)(mt * p.ntiles_n);
  const int grid = 8 * ((p.ntiles + 7) / 8);
  hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, GM>), dim3(grid), dim3(NTHREADS), 0, s, p);
  return hipGetLastError();
}

template <int GM>
hipError_t launch_igemm_g(IgemmP& p, hipStream_t s) {
  static const int force_bm = getenv("LMS_IGEMM_BM") ? atoi(getenv("LMS_IGEMM_BM")) : 0;   // tuning aid
  const int bn = p.nout <= 32 ? 32 : (p.nout <= 64 ? 64 : 128);
  long long red_total = (long long)p.taps * p.red;
  if (GM == GM_TRC) {                        // the longest reduction of a residue class
    red_total = p.red;
    for (int d = 0; d < 3; ++d) red_total *= (p.filt[d] + p.stride[d] - 1) / p.stride[d];
  }
  // bandwidth-bound layers (every 1x1, and 3x3 up to 256 channels) do better with more, smaller work-groups; swept on
  // whole ResNet-50 steps: thresholds 256 / 640 / 1200 / 2400 / none give 17.49 / 17.36 / 17.27 / 17.28 / 17.32 ms at batch 256
  int bm = red_total <= 2400 ? 64 : 128;
  if (force_bm) bm = force_bm;
  if (GM == GM_SMALL) bm = 128;
  if (bn == 32) return launch_igemm_t<128, 32, 4, 1, GM>(p, s);
  if (bn == 64) return bm == 64 ? launch_igemm_t<64, 64, 2, 2, (GM == GM_SMALL ? GM_FWD : GM)>(p, s) : launch_igemm_t<128, 64, 2, 2, GM>(p, s);
  return bm == 64 ? launch_igemm_t<64, 128, 2, 2, (GM == GM_SMALL ? GM_FWD : GM)>(p, s) : launch_igemm_t<128, 128, 2, 2, GM>(p, s);
}

// Tile and gather-mode choice depend on the shape only (never on addresses or memory pressure: runs must be repeatable).
hipError_t launch_igemm(IgemmP& p, hipStream_t s) {
  static const bool no_halo = getenv("LMS_NO_HALO") != nullptr;   // tuning aid: force the per-tap gather kernel
  if (!no_halo && p.mode == 1 && rf_eligible(p)) return launch_rf(p, s);   // the forward pass takes this path before packing
  if (!no_halo && halo_eligible(p)) return launch_halo(p, s);
  if (p.small) return launch_igemm_g<GM_SMALL>(p, s);
  if (p.mode == 0) return launch_igemm_g<GM_FWD>(p, s);
  if (p.stride[0] == 1 && p.stride[1] == 1 && p.stride[2] == 1) return launch_igemm_g<GM_TR1>(p, s);
  static const bool no_trc = getenv("LMS_NO_TRC") != nullptr;     // tuning aid: per-row residue checks instead of class tiles
  if (!no_trc && p.osp[0] % p.stride[0] == 0 && p.osp[1] % p.stride[1] == 0 && p.osp[2] % p.stride[2] == 0 && p.M > 0)
    return launch_igemm_g<GM_TRC>(p, s);
  return launch_igemm_g<GM_TRS>(p, s);
}

int small_jpad(const ConvGeom& g) { return cdiv((long long)g.taps() * g.c, BK) * BK; }

struct WgradSplit { int ctiles, ktiles, splits; long long rows_per_split; };
WgradSplit wgrad_split(long long rows, int taps, int cx, int ky) {
  WgradSplit w;
  w.ctiles = cdiv(cx, WG_T);
  w.ktiles = cdiv(ky, WG_T);
  const long long tiles = (long long)taps * w.ctiles * w.ktiles;
  const long long chunks = (rows + WG_T - 1) / WG_T;
  long long splits = (512 + tiles - 1) / tiles;   // about one resident work-group pair per CU
  if (splits > chunks) splits = chunks;
  if (splits < 1) splits = 1;
  const long long cps = (chunks + splits - 1) / splits;
  w.splits = (int)((chunks + cps - 1) / cps);
  w.rows_per_split = cps * WG_T;
  return w;
}

// Weight gradient of a 1x1 stride-1 convolution with at most 8 output channels (class heads): dw[c][k] = sum over
// positions of x[m][c] * dy[m][k].  No MFMA: a thread keeps 8 channels x 8 outputs of the sum in registers and
// walks over the rows of its work-group with a stride; threads of the same channel vector are then added in a
// fixed order (wave shuffles, then the four waves through LDS).  part[work-group][c][k].
constexpr int WT_WGS = 1024;
__global__ __launch_bounds__(256) void wgrad_tiny_kernel(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int ky,
                                                         long long rows_per_wg) {
  __shared__ float sh[4][64][8];                       // [wave][channel vector][...] one output column at a time
  const int cvn = cx >> 3;                             // a power of two, at most 64
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cv = tid & (cvn - 1), r = tid / cvn, rpb = 256 / cvn;
  const long long lo = (long long)blockIdx.x * rows_per_wg;
  const long long hi = lo + rows_per_wg < rows ? lo + rows_per_wg : rows;
  float acc[8][8];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[e][k] = 0.f;
  for (long long m = lo + r; m < hi; m += rpb) {
    const uint4 q = *reinterpret_cast<const uint4*>(X + m * cx + cv * 8);
    const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
    float xv[8], d[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) xv[e] = __uint_as_float((e & 1) ? (qw[e >> 1] & 0xffff0000u) : (qw[e >> 1] << 16));
    if (ky == 8 || ky == 4) {
      uint32_t dw4[4] = {0, 0, 0, 0};
      if (ky == 8) {
        const uint4 g = *reinterpret_cast<const uint4*>(DY + m * 8);
        dw4[0] = g.x; dw4[1] = g.y; dw4[2] = g.z; dw4[3] = g.w;
      } else {
        const uint2 g = *reinterpret_cast<const uint2*>(DY + m * 4);
        dw4[0] = g.x; dw4[1] = g.y;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = __uint_as_float((k & 1) ? (dw4[k >> 1] & 0xffff0000u) : (dw4[k >> 1] << 16));
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = k < ky ? bf2f(DY[m * ky + k]) : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[e][k] = __builtin_fmaf(xv[e], d[k], acc[e][k]);
  }
  // lanes with the same channel vector: lane, lane + cvn, ... ; add them pairwise at growing distance
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float v = acc[e][k];
      for (int dist = cvn; dist < 64; dist <<= 1) v += __shfl_xor(v, dist, 64);
      acc[e][k] = v;
    }
  float* out = part + (long long)blockIdx.x * cx * ky;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    if (k < ky) {                                       // uniform
      if (lane < cvn) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sh[wave][lane][e] = acc[e][k];
      }
      __syncthreads();
      if (tid < cvn * 8) {
        const int v = tid >> 3, e = tid & 7;
        out[(long long)(v * 8 + e) * ky + k] = (sh[0][v][e] + sh[1][v][e]) + (sh[2][v][e] + sh[3][v][e]);
      }
      __syncthreads();
    }
  }
}

bool wgrad_tiny_eligible(int cx, int ky, const int* filt, const int* stride, const int* pad) {
  static const bool off = getenv("LMS_NO_WGRAD_TINY") != nullptr;     // tuning aid
  for (int i = 0; i < 3; ++i)
    if (filt[i] != 1 || stride[i] != 1 || pad[i] != 0) return false;
  const int cvn = cx >> 3;
  return !off && ky <= 8 && (cx & 7) == 0 && cvn >= 1 && cvn <= 32 && (cvn & (cvn - 1)) == 0;
}
int wgrad_tiny_wgs(long long rows, int cx) {
  const long long per_iter = 256 / (cx >> 3);          // rows a work-group takes per iteration
  long long wgs = rows / (per_iter * 8);                // at least 8 iterations each
  return (int)(wgs < 1 ? 1 : (wgs > WT_WGS ? WT_WGS : wgs));
}

// First layers (1 to 4 channels): the segment kernel, unless the rows are shorter than its 64-position segments
// and the patch-tiled kernel for 3x3 stride-1 filters applies (small images: measured faster there).
bool wgrad_use_small(int cx, int ky, const int* asp, const int* osp, const int* filt, const int* stride) {
  if (!wgrad_small_eligible(cx, ky, asp, filt, stride)) return false;
  return osp[2] >= 64 || !wgrad_patch_eligible(cx, ky, filt, stride);
}

// The part of the workspace behind the partial filters: partial column sums of dy, [splits][ky].
float* colsum_part(void* ws, long long splits, long long per) { return reinterpret_cast<float*>(ws) + splits * per; }

hipError_t launch_wgrad_dw(const uint16_t* X, const uint16_t* DY, float* dw, void* ws, long long rows, int cx, int ky,
                           const int* asp, const int* osp, const int* filt, const int* stride, const int* pad,
                           int transpose, float* colsum_out, bool& colsum_done, hipStream_t s);

// colsum_out (or null): the sums of dy over all positions, per channel (the bias / shift gradient of the same
// layer).  The kernels that stage dy through registers add it up on the side; the others are followed by the plain
// column-sum pass, which reuses the workspace.
hipError_t launch_wgrad(const uint16_t* X, const uint16_t* DY, float* dw, void* ws, long long rows, int cx, int ky,
                        const int* asp, const int* osp, const int* filt, const int* stride, const int* pad,
                        int transpose, float* colsum_out, hipStream_t s) {
  bool done = false;
  hipError_t e = launch_wgrad_dw(X, DY, dw, ws, rows, cx, ky, asp, osp, filt, stride, pad, transpose, colsum_out, done, s);
  if (e != hipSuccess || !colsum_out || done) return e;
  return colsum(rows, ky, DY, colsum_out, ws, s);
}

hipError_t launch_wgrad_dw(const uint16_t* X, const uint16_t* DY, float* dw, void* ws, long long rows, int cx, int ky,
                           const int* asp, const int* osp, const int* filt, const int* stride, const int* pad,
                           int transpose, float* colsum_out, bool& colsum_done, hipStream_t s) {
  static const bool no_side = getenv("LMS_NO_WGRAD_COLSUM") != nullptr;   // tuning aid: always the separate pass
  const bool side = colsum_out && !no_side;
  if (!transpose && wgrad_tiny_eligible(cx, ky, filt, stride, pad)) {
    const int wgs = wgrad_tiny_wgs(rows, cx);
    const long long per_wg = (rows + wgs - 1) / wgs;
    hipLaunchKernelGGL(wgrad_tiny_kernel, dim3(wgs), dim3(256), 0, s, X, DY, reinterpret_cast<float*>(ws), rows, cx, ky, per_wg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long per = (long long)cx * ky;
    hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(cdiv(per / 4, 32)), dim3(256), 0, s, (const float4*)ws, (float4*)dw, per / 4, wgs);
    return hipGetLastError();
  }
  if (!transpose && wgrad_use_small(cx, ky, asp, osp, filt, stride)) {
    hipError_t e = launch_wgrad_small(X, DY, reinterpret_cast<float*>(ws), rows, cx, ky, asp, osp, filt, stride, pad, s);
    if (e != hipSuccess) return e;
    const long long per = (long long)filt[0] * filt[1] * filt[2] * cx * ky;
    hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(cdiv(per / 4, 32)), dim3(256), 0, s, (const float4*)ws, (float4*)dw, per / 4,
                       wgrad_small_splits(rows, osp));
    return hipGetLastError();
  }
  if (!transpose && wgrad_rows_eligible(cx, ky, filt, stride, pad)) {
    const long long per = (long long)cx * ky;
    const int splits = wgrad_rows_splits(rows, cx, ky);
    float* cs = side ? colsum_part(ws, splits, per) : nullptr;
    hipError_t e = launch_wgrad_rows(X, DY, reinterpret_cast<float*>(ws), rows, cx, ky, asp, osp, stride, cs, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(cdiv(per / 4, 32)), dim3(256), 0, s, (const float4*)ws, (float4*)dw, per / 4, splits);
    e = hipGetLastError();
    if (e != hipSuccess || !cs) return e;
    colsum_done = true;
    return col_reduce(cs, splits, ky, colsum_out, s);
  }
  static const bool no_patch = getenv("LMS_NO_WGRAD_PATCH") != nullptr;   // tuning aid
  if (!transpose && !no_patch && wgrad_patch_eligible(cx, ky, filt, stride)) {
    const long long batch = rows / ((long long)osp[0] * osp[1] * osp[2]);
    const int splits = wgrad_patch_splits(batch, asp, osp, filt, pad, cx, ky);
    const long long per = (long long)filt[0] * filt[1] * filt[2] * cx * ky;
    float* cs = side && wgrad_patch_colsum(filt, cx, ky) ? colsum_part(ws, splits, per) : nullptr;
    hipError_t e = launch_wgrad_patch(X, DY, reinterpret_cast<float*>(ws), batch, asp, osp, filt, pad, cx, ky, cs, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(cdiv(per / 4, 32)), dim3(256), 0, s, (const float4*)ws, (float4*)dw, per / 4, splits);
    e = hipGetLastError();
    if (e != hipSuccess || !cs) return e;
    colsum_done = true;
    return col_reduce(cs, splits, ky, colsum_out, s);
  }
  WgradP p{};
  p.X = X; p.DY = DY; p.part = reinterpret_cast<float*>(ws);
  p.M = rows; p.cx = cx; p.ky = ky;
  for (int i = 0; i < 3; ++i) { p.asp[i] = asp[i]; p.osp[i] = osp[i]; p.filt[i] = filt[i]; p.stride[i] = stride[i]; p.pad[i] = pad[i]; }
  p.taps = filt[0] * filt[1] * filt[2];
  WgradSplit w = wgrad_split(rows, p.taps, cx, ky);
  p.ctiles = w.ctiles; p.ktiles = w.ktiles; p.splits = w.splits; p.rows_per_split = w.rows_per_split;
  p.small = (cx & 7) != 0;
  const long long blocks = (long long)p.taps * w.ctiles * w.ktiles * w.splits;
  if (blocks > 0x7fffff00LL || rows >= 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(wgrad_kernel, dim3((unsigned)blocks), dim3(NTHREADS), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long per = (long long)p.taps * cx * ky;
  if (!transpose && (per & 3) == 0)
    hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(cdiv(per / 4, 32)), dim3(256), 0, s, (const float4*)p.part, (float4*)dw, per / 4, w.splits);
  else
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(cdiv(per, 256)), dim3(256), 0, s, p.part, dw, per, w.splits, p.taps, cx, ky, transpose);
  return hipGetLastError();
}

}  // namespace

uint64_t conv_fwd_ws(const ConvGeom& g) {
  if (g.c % 8 != 0) return (uint64_t)g.k * small_jpad(g) * 2;
  return (uint64_t)g.taps() * g.c * g.k * 2;
}
// Pointwise data gradient as a pointwise forward product: dx[m][c] = sum over k of dy[m][k] * wt[k][c] with the filter
// transposed (and scaled) into the workspace first, so the kernel that reads its filter as stored serves both.
// Taken where the layer widens (k > c, the gradient is reduced over more channels than it has): there it is 3 to
// 20 % faster than the general kernel on the ResNet-50 stages (186 -> 149 us for 512 -> 2048 on 7 x 7 positions at
// batch 852); where the layer narrows it is up to 40 % slower.
static bool dgrad_as_pw(const ConvGeom& g) {
  static const bool off = getenv("LMS_NO_DGRAD_PW") != nullptr;   // tuning aid
  if (off || g.taps() != 1 || (g.c & 7) != 0 || (g.k & 7) != 0 || g.c < 32 || g.k <= g.c) return false;
  for (int i = 0; i < 3; ++i)
    if (g.stride[i] != 1 || g.pad[i] != 0) return false;
  return true;
}

uint64_t conv_dgrad_ws(const ConvGeom& g, bool scaled) {
  if (g.k % 8 != 0) return (uint64_t)g.c * cdiv((long long)g.taps() * g.k, BK) * BK * 2;
  return (scaled || dgrad_as_pw(g)) ? (uint64_t)g.taps() * g.c * g.k * 2 : 0;
}
uint64_t conv_wgrad_ws(const ConvGeom& g, bool with_colsum) {
  WgradSplit w = wgrad_split(g.out_rows(), g.taps(), g.c, g.k);
  uint64_t splits = (uint64_t)w.splits;
  if (wgrad_tiny_eligible(g.c, g.k, g.filt, g.stride, g.pad)) {
    const uint64_t ts = (uint64_t)wgrad_tiny_wgs(g.out_rows(), g.c);
    if (ts > splits) splits = ts;
  }
  if (wgrad_use_small(g.c, g.k, g.in_sp, g.out_sp, g.filt, g.stride)) {
    const uint64_t ss = (uint64_t)wgrad_small_splits(g.out_rows(), g.out_sp);
    if (ss > splits) splits = ss;
  }
  if (wgrad_rows_eligible(g.c, g.k, g.filt, g.stride, g.pad)) {
    const uint64_t rs = (uint64_t)wgrad_rows_splits(g.out_rows(), g.c, g.k);
    if (rs > splits) splits = rs;
  }
  if (wgrad_patch_eligible(g.c, g.k, g.filt, g.stride)) {
    const uint64_t ps = (uint64_t)wgrad_patch_splits(g.n, g.in_sp, g.out_sp, g.filt, g.pad, g.c, g.k);
    static const bool no_patch = getenv("LMS_NO_WGRAD_PATCH") != nullptr;
    splits = no_patch ? (ps > splits ? ps : splits) : ps;
  }
  const uint64_t dw_part = splits * g.taps() * g.c * g.k * 4;
  if (!with_colsum) return dw_part;
  // partial column sums behind the partial filters, or the workspace of the separate column-sum pass
  const uint64_t side = dw_part + splits * g.k * 4, plain = reduce_ws(g.out_rows(), g.k);
  return side > plain ? side : plain;
}
uint64_t tconv_fwd_ws(const ConvGeom& g) { return (uint64_t)g.taps() * g.c * g.k * 2; }
uint64_t tconv_wgrad_ws(const ConvGeom& g) {
  WgradSplit w = wgrad_split(g.in_rows(), g.taps(), g.k, g.c);
  uint64_t splits = (uint64_t)w.splits;
  if (wgrad_rows_tconv_eligible(g.c, g.k, g.filt, g.stride)) {
    const uint64_t rs = (uint64_t)wgrad_rows_splits(g.in_rows(), g.c, g.taps() * g.k);
    if (rs > splits) splits = rs;
  }
  return splits * g.taps() * g.c * g.k * 4;
}

hipError_t conv_fwd(const ConvGeom& g, const void* x, const void* w, const Epilogue& ep, void* y, void* ws, hipStream_t s) {
  IgemmP p{};
  p.small = (g.c % 8) != 0;
  p.A = (const uint16_t*)x; p.B = (const uint16_t*)ws; p.out = (uint16_t*)y;
  p.scale = ep.scale; p.shift = ep.shift; p.add = (const uint16_t*)ep.add; p.mask = (const uint16_t*)ep.mask; p.relu = ep.relu;
  p.M = g.out_rows(); p.nout = g.k; p.red = g.c;
  fill_geom(g, p.asp, p.osp, p.filt, p.stride, p.pad);
  p.mode = 0;
  p.taps = g.taps();
  if (pw_eligible(p)) {        // pointwise: the filter is read as stored
    p.B = (const uint16_t*)w;
    return launch_pw(p, s);
  }
  if (rf_eligible(p)) {        // filter resident in registers: read as stored as well
    p.B = (const uint16_t*)w;
    return launch_rf(p, s);
  }
  if (conv_small_eligible(p)) {   // first layers with 1 to 4 channels: filter read as stored, patch matrix gathered in LDS
    p.B = (const uint16_t*)w;
    return launch_conv_small(p, s);
  }
  if (p.small) {
    p.jpad = small_jpad(g);
    const long long n = (long long)g.k * p.jpad;
    hipLaunchKernelGGL(pack_filter_small_kernel, dim3(cdiv(n, 256)), dim3(256), 0, s, (const uint16_t*)w, (uint16_t*)ws, g.taps(), g.c, g.k, p.jpad);
  } else {
    launch_pack_filter((const uint16_t*)w, nullptr, (uint16_t*)ws, g.taps(), g.c, g.k, 1, s);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_igemm(p, s);
}

// Data gradient of a 1x1 stride-1 convolution with at most 8 output channels (class heads): dx[m][c] = sum over k of
// dy[m][k] * w[c][k] (* scale[k], rounded to bf16 first like the packed filter of the general path).  Far too little
// arithmetic for the matrix unit: one thread per position and 8-channel vector, the filter slice in registers.
// A thread keeps one 8-channel vector of the filter and walks over `iters` positions: the filter slice is loaded once
// per thread, the index arithmetic is 32-bit and done once.  rpb = positions a block takes per iteration.
__global__ __launch_bounds__(256) void dgrad_tiny_kernel(IgemmP p, const float* kscale, int rpb, int iters) {
  const int cvn = p.nout >> 3;
  const int r = threadIdx.x / cvn, cv = threadIdx.x - r * cvn;
  if (r >= rpb) return;
  float wv[8][8];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      wv[e][k] = 0.f;
      if (k < p.red) {
        const uint16_t w = p.B[(cv * 8 + e) * p.red + k];
        wv[e][k] = kscale ? bf2f(f2bf(bf2f(w) * kscale[k])) : bf2f(w);
      }
    }
  const long long m0 = (long long)blockIdx.x * rpb * iters + r;
  EpiCoef none;
#pragma unroll 2
  for (int it = 0; it < iters; ++it) {
    const long long m = m0 + (long long)it * rpb;
    if (m >= p.M) return;
    float d[8];
    if (p.red == 8) {
      const uint4 q = *reinterpret_cast<const uint4*>(p.A + m * 8);
      const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = __uint_as_float((k & 1) ? (qw[k >> 1] & 0xffff0000u) : (qw[k >> 1] << 16));
    } else if (p.red == 4) {
      const uint2 q = *reinterpret_cast<const uint2*>(p.A + m * 4);
      const uint32_t qw[2] = {q.x, q.y};
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = k < 4 ? __uint_as_float((k & 1) ? (qw[k >> 1] & 0xffff0000u) : (qw[k >> 1] << 16)) : 0.f;
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = k < p.red ? bf2f(p.A[m * p.red + k]) : 0.f;
    }
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float a = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) a = __builtin_fmaf(d[k], wv[e][k], a);
      v[e] = a;
    }
    const long long off = m * p.nout + cv * 8;
    uint4 addq = make_uint4(0, 0, 0, 0), maskq = make_uint4(0, 0, 0, 0);
    if (p.add) addq = *reinterpret_cast<const uint4*>(p.add + off);
    if (p.mask) maskq = *reinterpret_cast<const uint4*>(p.mask + off);
    *reinterpret_cast<uint4*>(p.out + off) = epilogue_pack8(p, none, v, addq, maskq);
  }
}

hipError_t conv_dgrad(const ConvGeom& g, const void* dy, const void* w, const Epilogue& ep, void* dx, void* ws, hipStream_t s) {
  IgemmP p{};
  p.A = (const uint16_t*)dy; p.B = (const uint16_t*)w; p.out = (uint16_t*)dx;
  p.add = (const uint16_t*)ep.add; p.mask = (const uint16_t*)ep.mask; p.relu = ep.relu;
  p.M = g.in_rows(); p.nout = g.c; p.red = g.k;
  for (int i = 0; i < 3; ++i) {
    p.asp[i] = g.out_sp[i]; p.osp[i] = g.in_sp[i]; p.filt[i] = g.filt[i]; p.stride[i] = g.stride[i]; p.pad[i] = g.pad[i];
  }
  p.mode = 1;
  p.taps = g.taps();
  p.small = (g.k % 8) != 0;
  static const bool no_tiny = getenv("LMS_NO_DGRAD_TINY") != nullptr;     // tuning aid
  if (!no_tiny && g.taps() == 1 && g.k <= 8 && (g.c & 7) == 0 && g.c <= 2048 && g.stride[0] == 1 && g.stride[1] == 1 && g.stride[2] == 1 &&
      g.pad[0] == 0 && g.pad[1] == 0 && g.pad[2] == 0) {
    const int rpb = 256 / (g.c / 8);                    // positions per block and iteration
    long long iters = p.M / ((long long)rpb * 1024);    // about four blocks per compute unit, 4 to 32 positions per thread
    iters = iters < 4 ? 4 : (iters > 32 ? 32 : iters);
    const int blocks = cdiv(p.M, (long long)rpb * iters);
    hipLaunchKernelGGL(dgrad_tiny_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, ep.scale, rpb, (int)iters);
    return hipGetLastError();
  }
  if (dgrad_as_pw(g)) {
    launch_pack_filter((const uint16_t*)w, ep.scale, (uint16_t*)ws, 1, g.c, g.k, 1, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    p.B = (const uint16_t*)ws;
    p.mode = 0;
    p.small = false;
    if (pw_eligible(p)) return launch_pw(p, s);
    p.mode = 1;
    p.B = (const uint16_t*)w;
  }
  if (p.small) {
    // the reduction runs over the forward output channels: 16-byte loads need k % 8 == 0, otherwise
    // the (tap, k) index is flattened and gathered element by element
    p.jpad = cdiv((long long)g.taps() * g.k, BK) * BK;
    const long long n = (long long)g.c * p.jpad;
    hipLaunchKernelGGL(pack_filter_small_dgrad_kernel, dim3(cdiv(n, 256)), dim3(256), 0, s, (const uint16_t*)w, ep.scale, (uint16_t*)ws, g.taps(), g.c, g.k, p.jpad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    p.B = (const uint16_t*)ws;
  } else if (ep.scale) {
    launch_pack_filter((const uint16_t*)w, ep.scale, (uint16_t*)ws, g.taps(), g.c, g.k, 0, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    p.B = (const uint16_t*)ws;
  }
  return launch_igemm(p, s);
}

hipError_t conv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* dw, void* ws, hipStream_t s, float* colsum_out) {
  return launch_wgrad((const uint16_t*)x, (const uint16_t*)dy, dw, ws, g.out_rows(), g.c, g.k, g.in_sp, g.out_sp, g.filt,
                      g.stride, g.pad, 0, colsum_out, s);
}

// Transposed convolution (window = stride = 2): every output position takes exactly one filter tap,
// which is the transposed gather of a stride-2 convolution from the large grid to the small one.
hipError_t tconv_fwd(const ConvGeom& g, const void* x, const void* w, void* y, void* ws, hipStream_t s) {
  if (g.c % 8 != 0) return hipErrorInvalidValue;
  {   // window = stride: one pointwise product per tap, filter as stored (no packing pass)
    IgemmP q{};
    q.A = (const uint16_t*)x; q.B = (const uint16_t*)w; q.out = (uint16_t*)y;
    q.M = g.in_rows(); q.nout = g.k; q.red = g.c;
    bool same = true;
    for (int i = 0; i < 3; ++i) {
      q.asp[i] = g.in_sp[i]; q.osp[i] = g.out_sp[i]; q.filt[i] = 1; q.stride[i] = 1; q.pad[i] = 0;
      q.up[i] = g.stride[i];
      same = same && g.filt[i] == g.stride[i];
    }
    q.taps = 1;
    if (same && pw_up_eligible(q)) return launch_pw(q, s);
  }
  launch_pack_filter((const uint16_t*)w, nullptr, (uint16_t*)ws, g.taps(), g.c, g.k, 1, s);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  IgemmP p{};
  p.A = (const uint16_t*)x; p.B = (const uint16_t*)ws; p.out = (uint16_t*)y;
  p.M = g.out_rows(); p.nout = g.k; p.red = g.c;
  for (int i = 0; i < 3; ++i) {
    p.asp[i] = g.in_sp[i]; p.osp[i] = g.out_sp[i]; p.filt[i] = g.filt[i]; p.stride[i] = g.stride[i]; p.pad[i] = 0;
  }
  p.mode = 1;
  p.taps = g.taps();
  return launch_igemm(p, s);
}

hipError_t tconv_dgrad(const ConvGeom& g, const void* dy, const void* w, const Epilogue& ep, void* dx, hipStream_t s) {
  if (g.k % 8 != 0) return hipErrorInvalidValue;
  IgemmP p{};
  p.A = (const uint16_t*)dy; p.B = (const uint16_t*)w; p.out = (uint16_t*)dx;
  p.add = (const uint16_t*)ep.add; p.mask = (const uint16_t*)ep.mask;
  p.M = g.in_rows(); p.nout = g.c; p.red = g.k;
  for (int i = 0; i < 3; ++i) {
    p.asp[i] = g.out_sp[i]; p.osp[i] = g.in_sp[i]; p.filt[i] = g.filt[i]; p.stride[i] = g.stride[i]; p.pad[i] = 0;
  }
  p.mode = 0;
  p.taps = g.taps();
  return launch_igemm(p, s);
}

// dw[t][c][k] = sum over splits of part[split][c][t * kk + k], four k at a time: the sum of wgrad_reduce_vec_kernel
// (every thread adds one eighth of the splits, the eight partial sums are added in a fixed order), stored permuted.
__global__ __launch_bounds__(256) void wgrad_reduce_taps_kernel(const float4* part, float4* dw, int cx, int taps, int kk4, int splits) {
  __shared__ float4 sh[8][32];
  const long long per4 = (long long)cx * taps * kk4;
  const int o = threadIdx.x & 31, g = threadIdx.x >> 5;
  const long long idx = (long long)blockIdx.x * 32 + o;          // source order: [c][t][k]
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (idx < per4) {
    for (int i = g; i < splits; i += 8) {
      const float4 a = part[(long long)i * per4 + idx];
      s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
  }
  sh[g][o] = s;
  __syncthreads();
  if (g == 0 && idx < per4) {
    float4 t = sh[0][o];
#pragma unroll
    for (int j = 1; j < 8; ++j) { t.x += sh[j][o].x; t.y += sh[j][o].y; t.z += sh[j][o].z; t.w += sh[j][o].w; }
    const int k4 = (int)(idx % kk4);
    const long long r = idx / kk4;
    const int tp = (int)(r % taps);
    const int c = (int)(r / taps);
    dw[((long long)tp * cx + c) * kk4 + k4] = t;
  }
}

hipError_t tconv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* dw, void* ws, hipStream_t s) {
  bool exact = true;                                     // the output grid is the input grid times the stride
  for (int i = 0; i < 3; ++i) exact = exact && g.out_sp[i] == g.in_sp[i] * g.stride[i];
  if (exact && wgrad_rows_tconv_eligible(g.c, g.k, g.filt, g.stride)) {
    // window = stride: a pointwise weight gradient over the positions of x against taps * k gathered channels of dy
    hipError_t e = launch_wgrad_rows_tconv((const uint16_t*)x, (const uint16_t*)dy, reinterpret_cast<float*>(ws), g.in_rows(), g.c, g.k,
                                           g.in_sp, g.out_sp, g.stride, s);
    if (e != hipSuccess) return e;
    const int taps = g.taps(), kk4 = g.k / 4;
    const long long per = (long long)g.c * taps * kk4;
    hipLaunchKernelGGL(wgrad_reduce_taps_kernel, dim3((unsigned)cdiv(per, 32)), dim3(256), 0, s, (const float4*)ws, (float4*)dw, g.c, taps, kk4,
                       wgrad_rows_splits(g.in_rows(), g.c, taps * g.k));
    return hipGetLastError();
  }
  // gathered operand: dy on the large grid (channels k); plain operand: x (channels c); result [tap][k][c] -> transpose
  int zero[3] = {0, 0, 0};
  return launch_wgrad((const uint16_t*)dy, (const uint16_t*)x, dw, ws, g.in_rows(), g.k, g.c, g.out_sp, g.in_sp, g.filt,
                      g.stride, zero, 1, nullptr, s);
}

}  // namespace lms
