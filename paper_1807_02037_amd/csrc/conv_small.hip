// Forward convolution with very few input channels (first layers: 3 or 1 channels), any filter, stride and
// padding, 2-D or 3-D, up to 64 output channels.
//
// The reduction index is j = (tap, channel) flattened (147 for a 7x7 filter on 3 channels).  The whole filter
// [j][k] is read as stored, staged through LDS once per work-group and kept in registers as MFMA fragments.  A
// work-group then walks over output row segments (64 consecutive positions of one output row): it gathers the
// transposed patch matrix P^T[j][position] into LDS (input rows first, with coalesced loads issued one segment ahead, then one 2-byte LDS
// element per lane and row j, at offsets kept in registers), and multiplies with both operands fetched by the LDS
// transpose read.  The kernel is a template on the reduction length and on the loads per staged input row, so the
// work per segment is straight-line code.  Products are taken transposed, so a lane ends up with consecutive output channels of one
// position and stores 16-byte vectors straight from the accumulators.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"
#include "small_gather.hpp"

namespace lms {

namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int CS_ROWS = 64;            // positions per segment
constexpr int CS_JMAX = 160;           // (taps x channels) at most, padded to a multiple of 16
constexpr int CS_LDP = 96;             // pitch of P^T rows and of the staged filter rows (192 bytes: 64 modulo 256)

struct CSmallP {
  IgemmP g;
  int J;
  int segs;                    // segments per output row
  long long stages;            // batch * osp[0] * osp[1] * segs
  long long stages_per_wg;
};

__device__ __forceinline__ bf16x8 cs_tr_frag(const uint16_t* p0, const uint16_t* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p0);
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p1);
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// KS: reduction steps of 16 (tap, channel) pairs; NH: loads per lane and staged row.
template <int KS, int NH>
__global__ __launch_bounds__(NTHREADS, 2) void conv_small_kernel(CSmallP cp) {
  constexpr int JP = KS * 16;
  __shared__ __attribute__((aligned(16))) uint16_t sP[JP * CS_LDP];
  __shared__ uint16_t raw[SG_RAW_EL];
  const IgemmP& p = cp.g;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int src_off = (li >> 2) * CS_LDP + 16 * (lg & 1) + 4 * (li & 3);
  const int half = lg >> 1;
  const int ut = wave & 1, kt = wave >> 1;                  // this wave's 32 positions x 32 channels
  const bool has_tile = kt * 32 < p.nout;

  int code[JP / 4];                      // offsets of this wave's P^T rows in the staged input rows
  SgRows rw;
  sg_rows_init(rw, p.filt);
  sg_codes(code, cp.J, p.red, p.filt);
  // ---- the filter [j][k] as stored, zero beyond J and beyond the output channels; then this wave's fragments ----
  for (int v = tid; v < SG_RAWP; v += NTHREADS) raw[SG_RMAX * SG_RAWP + v] = 0;
  for (int v = tid; v < JP * 8; v += NTHREADS) {
    const int j = v >> 3, cv = v & 7;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (j < cp.J && cv * 8 < p.nout) w = *reinterpret_cast<const uint4*>(p.B + (long long)j * p.nout + cv * 8);
    *reinterpret_cast<uint4*>(sP + j * CS_LDP + cv * 8) = w;
  }
  __syncthreads();
  bf16x8 wf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const uint16_t* q = sP + (ks * 16 + 8 * half) * CS_LDP + kt * 32 + src_off;
    wf[ks] = cs_tr_frag(q, q + 4 * CS_LDP);
  }

  EpiCoef coef[2];
#pragma unroll
  for (int pr = 0; pr < 2; ++pr) {
    const int n = kt * 32 + pr * 16 + (lane >> 5) * 8;
    if (n < p.nout) epilogue_coef(p, n, 8, coef[pr]);
  }

  const long long s_begin = (long long)blockIdx.x * cp.stages_per_wg;
  const long long s_end = (s_begin + cp.stages_per_wg < cp.stages) ? s_begin + cp.stages_per_wg : cp.stages;
  // output row (nb, od, oh) and segment of the first stage; stepped from there
  int seg = (int)(s_begin % cp.segs);
  long long r0 = s_begin / cp.segs;
  int oh = (int)(r0 % p.osp[1]); r0 /= p.osp[1];
  int od = (int)(r0 % p.osp[0]);
  long long nb = r0 / p.osp[0];
  // the input rows of a segment are requested one segment ahead: they arrive while the previous one is multiplied
  SgRegs<NH> rows_next;
  if (s_begin < s_end) sg_load_rows<NH>(rows_next, p.A, rw, nb, od, oh, seg * CS_ROWS, p.asp, p.stride, p.pad, p.filt, p.red);
  // The results of a segment are stored one segment late, right after the wait for the staged rows: loads and
  // stores share one counter whose waits are all-or-nothing once both kinds are pending, so a store issued at the end
  // of a segment would be waited for, with its full latency, at the start of the next.
  uint4 out_prev[2];
  long long off_prev[2] = {-1, -1};
  auto flush_prev = [&]() {
#pragma unroll
    for (int pr = 0; pr < 2; ++pr)
      if (off_prev[pr] >= 0) epilogue_put8(p, out_prev[pr], 8, off_prev[pr], true);
  };
  for (long long st = s_begin; st < s_end; ++st) {
    const long long r = (nb * p.osp[0] + od) * p.osp[1] + oh;
    const int ow0 = seg * CS_ROWS;
    const int valid = (p.osp[2] - ow0) < CS_ROWS ? (p.osp[2] - ow0) : CS_ROWS;
    if (++seg == cp.segs) {
      seg = 0;
      if (++oh == p.osp[1]) {
        oh = 0;
        if (++od == p.osp[0]) { od = 0; ++nb; }
      }
    }

    __syncthreads();                                    // the previous segment (or the filter) is fully consumed
    // ---- P^T of the segment: input rows to LDS, then gathered ----
    sg_store_rows<NH>(raw, rows_next, p.filt);
    flush_prev();
    off_prev[0] = off_prev[1] = -1;
    if (st + 1 < s_end) sg_load_rows<NH>(rows_next, p.A, rw, nb, od, oh, seg * CS_ROWS, p.asp, p.stride, p.pad, p.filt, p.red);
    __syncthreads();
    sg_build_pt(sP, CS_LDP, raw, code, p.stride[2] * p.red);
    __syncthreads();
    if (!has_tile) continue;
    // ---- y^T[k][position] = sum over j of w[j][k] * P^T[j][position] ----
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint16_t* q = sP + (ks * 16 + 8 * half) * CS_LDP + ut * 32 + src_off;
      const bf16x8 af = cs_tr_frag(q, q + 4 * CS_LDP);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks], af, acc, 0, 0, 0);
    }
    // ---- epilogue: a lane holds 16 channels of one position, 4 consecutive ones per register group with the
    // half-waves interleaved; one cross-half swap per register pair leaves 8 consecutive channels per lane ----
    const int u = ut * 32 + (lane & 31);
    const long long row_off = (r * p.osp[2] + ow0 + u) * p.nout;
    uint4 outw[2];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      float v[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[8 * pr + e]), __float_as_uint(acc[8 * pr + 4 + e]), false, false);
        v[e] = __uint_as_float(sw[0]);
        v[4 + e] = __uint_as_float(sw[1]);
      }
      const int n = kt * 32 + pr * 16 + (lane >> 5) * 8;
      outw[pr] = make_uint4(0, 0, 0, 0);
      if (u >= valid || n >= p.nout) continue;
      uint4 addq = make_uint4(0, 0, 0, 0), maskq = make_uint4(0, 0, 0, 0);
      if (p.add) addq = *reinterpret_cast<const uint4*>(p.add + row_off + n);
      if (p.mask) maskq = *reinterpret_cast<const uint4*>(p.mask + row_off + n);
      outw[pr] = epilogue_pack8(p, coef[pr], v, addq, maskq);
    }
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const int n = kt * 32 + pr * 16 + (lane >> 5) * 8;
      out_prev[pr] = outw[pr];
      off_prev[pr] = (u < valid && n < p.nout) ? row_off + n : -1;
    }
  }
  flush_prev();
}

template <int KS>
void cs_launch(int nh, dim3 grid, dim3 block, hipStream_t s, const CSmallP& cp) {
  if (nh == 2) hipLaunchKernelGGL((conv_small_kernel<KS, 2>), grid, block, 0, s, cp);
  else if (nh == 4) hipLaunchKernelGGL((conv_small_kernel<KS, 4>), grid, block, 0, s, cp);
  else hipLaunchKernelGGL((conv_small_kernel<KS, 8>), grid, block, 0, s, cp);
}

}  // namespace

bool conv_small_eligible(const IgemmP& p) {
  static const bool off = getenv("LMS_NO_CONV_SMALL") != nullptr;      // tuning aid
  if (off || p.mode != 0 || (p.red & 7) == 0 || p.red > 4) return false;
  const int J = p.filt[0] * p.filt[1] * p.filt[2] * p.red;
  if (J > CS_JMAX || p.nout > 64 || (p.nout & 7) != 0) return false;
  return sg_fits(p.asp, p.filt, p.stride, p.red);
}

hipError_t launch_conv_small(IgemmP& p, hipStream_t s) {
  static const int force = getenv("LMS_CONV_SMALL_WGS") ? atoi(getenv("LMS_CONV_SMALL_WGS")) : 0;   // tuning aid
  CSmallP cp{};
  cp.g = p;
  cp.J = p.filt[0] * p.filt[1] * p.filt[2] * p.red;
  cp.segs = (p.osp[2] + CS_ROWS - 1) / CS_ROWS;
  cp.stages = p.M / p.osp[2] * cp.segs;
  if (cp.stages <= 0) return hipSuccess;
  long long wgs = force > 0 ? force : 1024;            // a work-group stages the filter once, then takes a run of segments
  if (wgs > cp.stages) wgs = cp.stages;
  cp.stages_per_wg = (cp.stages + wgs - 1) / wgs;
  wgs = (cp.stages + cp.stages_per_wg - 1) / cp.stages_per_wg;
  const int ks = (cp.J + 15) / 16, nh = sg_loads(p.filt, p.stride, p.red);
  const dim3 grid((unsigned)wgs), block(NTHREADS);
  // instantiated reduction lengths; a shorter reduction runs the next longer one with rows of zeros
  if (ks <= 2) cs_launch<2>(nh, grid, block, s, cp);
  else if (ks <= 4) cs_launch<4>(nh, grid, block, s, cp);
  else if (ks <= 7) cs_launch<7>(nh, grid, block, s, cp);
  else cs_launch<10>(nh, grid, block, s, cp);
  return hipGetLastError();
}

}  // namespace lms
