// Weight gradient of convolutions with very few input channels (first layers: 3 or 1 channels), any filter,
// stride and padding, 2-D or 3-D.
//
// With so few channels the filter gradient is small: dw[j][k] with j = (tap, channel) flattened (147 for a 7x7
// filter on 3 channels) and k up to 64 output channels.  A work-group owns the whole of it and walks over a range
// of output row segments (64 consecutive positions of one output row).  Per segment it gathers the transposed
// patch matrix P^T[j][position] into LDS (input rows first, with coalesced loads, then one 2-byte LDS element per
// lane and row j), copies the 64 x k tile of the output gradient next to it, and multiplies:
// the reduction runs over positions, P^T rows give one operand with 16-byte reads, the gradient tile gives the
// other through the LDS transpose read.  The output gradient is read once in total (the per-tap kernel reads it
// once per tap).  Partial sums per work-group go to the split buffer and are summed in a fixed order.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "kernels.hpp"
#include "conv_common.hpp"
#include "small_gather.hpp"

namespace lms {

namespace {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int WS_ROWS = 64;            // positions per segment
constexpr int WS_JMAX = 160;           // (taps x channels) at most, padded to a multiple of 32
constexpr int WS_LDP = WS_ROWS + 8;    // pitch of P^T rows (144 bytes: conflict-free 16-byte reads)
constexpr int WS_LDY = 96;             // pitch of the gradient tile rows (64 channels + 32: 64 bytes modulo 256)

struct WSmallP {
  const uint16_t* X;
  const uint16_t* DY;
  float* part;
  int cx, ky, J;
  int asp[3], osp[3], filt[3], stride[3], pad[3];
  int segs;                    // segments per output row
  long long stages;            // batch * osp[0] * osp[1] * segs
  long long stages_per_split;
  int splits;
};

__device__ __forceinline__ bf16x8 ws_tr_frag(const uint16_t* p0, const uint16_t* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p0);
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p1);
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// JT: 32-row tiles of (tap, channel) pairs; NH: loads per lane and staged row.
template <int JT, int NH>
__global__ __launch_bounds__(NTHREADS, 2) void wgrad_small_kernel(WSmallP p) {
  constexpr int JP = JT * 32;
  constexpr int WS_MAXT = (JT * 2 + 3) / 4;     // MFMA tiles per wave at most (JT x 2 tiles over 4 waves)
  __shared__ __attribute__((aligned(16))) uint16_t sP[JP * WS_LDP];
  __shared__ __attribute__((aligned(16))) uint16_t sY[WS_ROWS * WS_LDY];
  __shared__ uint16_t raw[SG_RAW_EL];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int KT = (p.ky + 31) / 32;

  int code[JP / 4];                      // offsets of this wave's P^T rows in the staged input rows
  SgRows rw;
  sg_rows_init(rw, p.filt);
  sg_codes(code, p.J, p.cx, p.filt);
  for (int v = tid; v < SG_RAWP; v += NTHREADS) raw[SG_RMAX * SG_RAWP + v] = 0;

  // MFMA tiles of this wave: tile t = wave + 4q -> (jt, kt)
  int t_j[WS_MAXT], t_k[WS_MAXT];
  int ntile = 0;
#pragma unroll
  for (int q = 0; q < WS_MAXT; ++q) {
    const int t = wave + 4 * q;
    t_j[q] = 0; t_k[q] = 0;
    if (t < JT * KT) { t_j[q] = t / KT; t_k[q] = t % KT; ntile = q + 1; }
  }
  f32x16 acc[WS_MAXT];
#pragma unroll
  for (int q = 0; q < WS_MAXT; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;

  const int li = lane & 15, lg = lane >> 4;
  const int src_off = (li >> 2) * WS_LDY + 16 * (lg & 1) + 4 * (li & 3);
  const int half = lg >> 1;

  const long long s_begin = (long long)blockIdx.x * p.stages_per_split;
  const long long s_end = (s_begin + p.stages_per_split < p.stages) ? s_begin + p.stages_per_split : p.stages;
  const int yv = p.ky >> 3;             // 16-byte vectors per gradient row

  // output row (nb, od, oh) and segment of the first stage; stepped from there
  int seg = (int)(s_begin % p.segs);
  long long r0 = s_begin / p.segs;
  int oh = (int)(r0 % p.osp[1]); r0 /= p.osp[1];
  int od = (int)(r0 % p.osp[0]);
  long long nb = r0 / p.osp[0];
  // both operands of a segment are requested one segment ahead: they arrive while the previous one is multiplied
  constexpr int YV = WS_ROWS * 8 / NTHREADS;      // gradient vectors per thread
  SgRegs<NH> rows_next;
  uint4 dy_next[YV];
  auto load_dy = [&](long long row, int w0) {
    const int ok = (p.osp[2] - w0) < WS_ROWS ? (p.osp[2] - w0) : WS_ROWS;
#pragma unroll
    for (int i = 0; i < YV; ++i) {
      const int v = tid + i * NTHREADS, q = v >> 3, cv = v & 7;
      dy_next[i] = make_uint4(0, 0, 0, 0);
      if (q < ok && cv < yv) dy_next[i] = *reinterpret_cast<const uint4*>(p.DY + ((row * p.osp[2] + w0 + q) * p.ky) + cv * 8);
    }
  };
  if (s_begin < s_end) {
    load_dy((nb * p.osp[0] + od) * p.osp[1] + oh, seg * WS_ROWS);
    sg_load_rows<NH>(rows_next, p.X, rw, nb, od, oh, seg * WS_ROWS, p.asp, p.stride, p.pad, p.filt, p.cx);
  }
  for (long long st = s_begin; st < s_end; ++st) {
    if (++seg == p.segs) {
      seg = 0;
      if (++oh == p.osp[1]) {
        oh = 0;
        if (++od == p.osp[0]) { od = 0; ++nb; }
      }
    }

    __syncthreads();                                    // the previous segment is fully consumed
    // ---- gradient tile: 64 positions x ky channels, zero beyond the row end and beyond ky ----
#pragma unroll
    for (int i = 0; i < YV; ++i) {
      const int v = tid + i * NTHREADS;
      *reinterpret_cast<uint4*>(sY + (v >> 3) * WS_LDY + (v & 7) * 8) = dy_next[i];
    }
    // ---- P^T of the segment: input rows to LDS, then gathered ----
    sg_store_rows<NH>(raw, rows_next, p.filt);
    if (st + 1 < s_end) {
      load_dy((nb * p.osp[0] + od) * p.osp[1] + oh, seg * WS_ROWS);
      sg_load_rows<NH>(rows_next, p.X, rw, nb, od, oh, seg * WS_ROWS, p.asp, p.stride, p.pad, p.filt, p.cx);
    }
    __syncthreads();
    sg_build_pt(sP, WS_LDP, raw, code, p.stride[2] * p.cx);
    __syncthreads();
    // ---- dw[j][k] += sum over the 64 positions ----
#pragma unroll
    for (int ks = 0; ks < WS_ROWS / 16; ++ks) {
      const int q0 = ks * 16 + 8 * half;
#pragma unroll
      for (int q = 0; q < WS_MAXT; ++q) {
        if (q < ntile) {
          const bf16x8 af = *reinterpret_cast<const bf16x8*>(sP + (t_j[q] * 32 + (lane & 31)) * WS_LDP + q0);
          const uint16_t* yb = sY + q0 * WS_LDY + t_k[q] * 32 + src_off;
          const bf16x8 bfr = ws_tr_frag(yb, yb + 4 * WS_LDY);
          acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr, acc[q], 0, 0, 0);
        }
      }
    }
  }

  float* out = p.part + (long long)blockIdx.x * p.J * p.ky;
#pragma unroll
  for (int q = 0; q < WS_MAXT; ++q) {
    if (q >= ntile) continue;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int j = t_j[q] * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      const int k = t_k[q] * 32 + (lane & 31);
      if (j < p.J && k < p.ky) out[(long long)j * p.ky + k] = acc[q][v];
    }
  }
}

long long ws_stages(long long rows, const int* osp) {
  const int segs = (osp[2] + WS_ROWS - 1) / WS_ROWS;
  return rows / osp[2] * segs;
}

template <int JT>
void ws_launch(int nh, dim3 grid, dim3 block, hipStream_t s, const WSmallP& p) {
  if (nh == 2) hipLaunchKernelGGL((wgrad_small_kernel<JT, 2>), grid, block, 0, s, p);
  else if (nh == 4) hipLaunchKernelGGL((wgrad_small_kernel<JT, 4>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((wgrad_small_kernel<JT, 8>), grid, block, 0, s, p);
}

}  // namespace

bool wgrad_small_eligible(int cx, int ky, const int* asp, const int* filt, const int* stride) {
  static const bool off = getenv("LMS_NO_WGRAD_SMALL") != nullptr;     // tuning aid
  const int J = filt[0] * filt[1] * filt[2] * cx;
  if (off || (cx & 7) == 0 || cx > 4) return false;
  if (J > WS_JMAX || ky > 64 || (ky & 7) != 0) return false;
  return sg_fits(asp, filt, stride, cx);
}

int wgrad_small_splits(long long rows, const int* osp) {
  static const int force = getenv("LMS_WGRAD_SMALL_WGS") ? atoi(getenv("LMS_WGRAD_SMALL_WGS")) : 0;   // tuning aid
  const long long stages = ws_stages(rows, osp);
  long long target = force > 0 ? force : 512;                          // two work-groups per compute unit
  if (target > stages) target = stages;
  if (target < 1) target = 1;
  const long long per = (stages + target - 1) / target;
  return (int)((stages + per - 1) / per);
}

hipError_t launch_wgrad_small(const uint16_t* X, const uint16_t* DY, float* part, long long rows, int cx, int ky, const int* asp,
                              const int* osp, const int* filt, const int* stride, const int* pad, hipStream_t s) {
  WSmallP p{};
  p.X = X; p.DY = DY; p.part = part;
  p.cx = cx; p.ky = ky; p.J = filt[0] * filt[1] * filt[2] * cx;
  for (int i = 0; i < 3; ++i) { p.asp[i] = asp[i]; p.osp[i] = osp[i]; p.filt[i] = filt[i]; p.stride[i] = stride[i]; p.pad[i] = pad[i]; }
  p.segs = (osp[2] + WS_ROWS - 1) / WS_ROWS;
  p.stages = ws_stages(rows, osp);
  p.splits = wgrad_small_splits(rows, osp);
  p.stages_per_split = (p.stages + p.splits - 1) / p.splits;
  if (p.stages <= 0) return hipSuccess;
  const int jt = (p.J + 31) / 32, nh = sg_loads(filt, stride, cx);
  const dim3 grid(p.splits), block(NTHREADS);
  // instantiated row-tile counts; fewer rows run the next larger one with rows of zeros
  if (jt <= 1) ws_launch<1>(nh, grid, block, s, p);
  else if (jt <= 2) ws_launch<2>(nh, grid, block, s, p);
  else if (jt <= 3) ws_launch<3>(nh, grid, block, s, p);
  else ws_launch<5>(nh, grid, block, s, p);
  return hipGetLastError();
}

}  // namespace lms
