// Executor: runs a (rewritten) graph inside a caller-supplied arena whose size is the memory budget.
//
// Mirrors the execution model of Sections 3.2-3.5: an operation runs once its data and control
// inputs are done; a tensor's memory is released after its last consumer (reference counting,
// 3.5); a swap-out is the identity placed on the host, i.e. a device-to-host copy issued right
// after its producer, a swap-in a host-to-device copy that may start once its control operation
// has finished (4.2.1).  Compute kernels run on one in-order stream, the two copy directions on
// their own streams; all ordering between streams is expressed with events planned once, together
// with every tensor's arena offset (shapes are static).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "graph.hpp"
#include "kernels.hpp"

namespace lms {

namespace {

ConvGeom geom_of(const Node& xin, const Node& yout, const lms_attr& a, bool is_tconv) {
  ConvGeom g;
  const int nsp = xin.nsp();
  g.n = xin.dims[0];
  g.c = (int)xin.channels();
  g.k = (int)yout.channels();
  for (int i = 0; i < nsp; ++i) {
    const int ax = 3 - nsp + i;
    g.in_sp[ax] = (int)xin.dims[1 + i];
    g.out_sp[ax] = (int)yout.dims[1 + i];
    g.filt[ax] = is_tconv ? 2 : a.filt[i];
    g.stride[ax] = is_tconv ? 2 : a.stride;
    g.pad[ax] = is_tconv ? 0 : a.pad;
  }
  return g;
}

}  // namespace

namespace {
// The operation a tensor comes from, through any swap-out / swap-in pairs.
int tensor_origin(const Graph& g, int v) {
  while (g.nodes[v].op == LMS_OP_SWAP_IN || g.nodes[v].op == LMS_OP_SWAP_OUT) v = g.nodes[v].in[0];
  return v;
}
constexpr int PAIR_WINDOW = 8;   // the backward builder emits a layer's weight gradient and its column sum within a few ids
}  // namespace

int colsum_host_wgrad(const Graph& g, int c) {
  const Node& nc = g.nodes[c];
  if (nc.op != LMS_OP_COLSUM || !nc.external || nc.in.size() != 1) return -1;
  const int dz = tensor_origin(g, nc.in[0]);
  if (g.nodes[dz].dtype != LMS_BF16) return -1;
  for (int w = c - 1; w >= 0 && w >= c - PAIR_WINDOW; --w) {
    const Node& nw = g.nodes[w];
    if (nw.op == LMS_OP_CONV_WGRAD && tensor_origin(g, nw.in[1]) == dz) return w;
  }
  return -1;
}

int wgrad_side_colsum(const Graph& g, int w) {
  if (g.nodes[w].op != LMS_OP_CONV_WGRAD) return -1;
  const int n = (int)g.nodes.size();
  for (int c = w + 1; c < n && c <= w + PAIR_WINDOW; ++c)
    if (g.nodes[c].op == LMS_OP_COLSUM && colsum_host_wgrad(g, c) == w) return c;
  return -1;
}

uint64_t workspace_bytes(const Graph& g, const Node& n) {
  auto IN = [&](int i) -> const Node& { return g.nodes[n.in[i]]; };
  switch (n.op) {
    case LMS_OP_CONV: return conv_fwd_ws(geom_of(IN(0), n, n.attr, false));
    case LMS_OP_CONV_DGRAD: return conv_dgrad_ws(geom_of(n, IN(0), n.attr, false), (n.attr.flags & LMS_F_AFFINE) != 0);
    case LMS_OP_CONV_WGRAD: return conv_wgrad_ws(geom_of(IN(0), IN(1), n.attr, false), wgrad_side_colsum(g, n.id) >= 0);
    case LMS_OP_TCONV: return tconv_fwd_ws(geom_of(IN(0), n, n.attr, true));
    case LMS_OP_TCONV_WGRAD: return tconv_wgrad_ws(geom_of(IN(0), IN(1), n.attr, true));
    case LMS_OP_MSE: return reduce_ws(0, 0);
    case LMS_OP_SOFTMAX_CE: return reduce_ws(IN(0).channels() > 64 ? IN(0).numel() / IN(0).channels() : 0, 0);
    case LMS_OP_COLSUM:
      if (colsum_host_wgrad(g, n.id) >= 0) return 0;       // comes out of the weight-gradient pass
      return reduce_ws(IN(0).numel() / IN(0).channels(), (int)IN(0).channels());
    default: return 0;
  }
}

constexpr int64_t STAGE_SLOTS = 8192;       // slots per staging buffer (32 MiB of tensor, 36 MB of buffer)
constexpr int STAGE_BUFS = 2;               // staging buffers per direction: one per lane of a staged swap
uint64_t swap_staging_bytes() { return 2 * (uint64_t)STAGE_BUFS * STAGE_SLOTS * swap_slot_stride(); }

struct Exec {
  Graph g;
  PlanResult plan;
  char* arena = nullptr;
  uint64_t arena_bytes = 0;
  char* pinned = nullptr;
  uint64_t pinned_bytes = 0;
  hipStream_t s_compute = nullptr, s_d2h = nullptr, s_h2d = nullptr;
  uint32_t flags = 0;
  std::vector<void*> bound;
  std::vector<hipEvent_t> ev;                 // event recorded after a node, where another stream needs it
  std::vector<std::vector<int>> waits;        // nodes whose events a node's stream waits for first
  std::vector<std::vector<int>> poison_waits; // extra waits before poisoning the blocks released after a node
  std::vector<std::vector<int>> dying;        // blocks released after a node (by position)
  hipEvent_t join_d2h = nullptr, join_h2d = nullptr;
  uint64_t bytes_d2h = 0, bytes_h2d = 0;
  int n_kernels = 0, n_copies = 0;
  // Updates held back to go out in one launch (sgd_update_batch): node ids, and a mark on every node a later
  // operation must not touch before they have run (the updated variable, the update itself).
  std::vector<int> pending;
  std::vector<char> pend_mark;
  int copy_blocks = 64;     // work-groups of a swap copy kernel
  // work-groups of the encoding / decoding swap kernels.  Kernels that drive the host link slow the convolutions
  // running beside them down once the link saturates (a 1x1 convolution beside a decoder: unchanged up to 128
  // work-groups, 1.6 times longer at 512; beside an encoder: unchanged up to 96, 1.4 times longer from 112 on), and a
  // copy engine does not (hipMemcpyAsync beside the same convolution: unchanged).  The decoder reaches 51 GB/s with 128
  // work-groups; the encoder needs the saturated link for its 52 GB/s (42 GB/s at 96), and on the swapped ResNet-50
  // steps the faster swap-outs win at every batch (batch 1278: 100.8 ms with 512 work-groups, 105.2 with 96; batch
  // 3796: 802 against 866 ms).
  int encode_blocks = 512, decode_blocks = 160;
  bool encodes(const Node& n) const {
    return (flags & LMS_X_ENCODE_SWAPS) && !(flags & LMS_X_DMA_COPY) && swap_is_encodable(n);
  }
  bool events_ok = true;   // an event that could not be created would silently drop an ordering between streams
  // LMS_X_TIMING: timing events, all created with the executor.  Per compute node that waits for a side stream, one
  // event before and one after the waits (the gap is the time the compute stream stood still); per copy, one before
  // and one after it on its side stream; one at each end of the step on the compute stream.
  struct WaitSpan { hipEvent_t before = nullptr, after = nullptr; bool on_h2d = false, on_d2h = false; };
  std::vector<WaitSpan> wait_span;            // per node
  std::vector<hipEvent_t> copy_begin, copy_end;   // per node (swap operations on a side stream)
  hipEvent_t step_begin = nullptr, step_end = nullptr;
  uint64_t last_enc_d2h = 0, last_enc_h2d = 0;    // encoded bytes counted after the latest synchronised step
  // LMS_X_STAGED_SWAPS: staging buffers at the end of the arena (STAGE_BUFS per direction, STAGE_SLOTS slots each) and, per
  // swap-out node, the staged width chosen after the latest synchronised step (0: direct transfer)
  char* stage_out = nullptr;
  char* stage_in = nullptr;
  std::vector<int> stage_w;
  hipEvent_t stage_start[2] = {nullptr, nullptr};   // per direction: the node's stream has waited for its dependencies
  hipEvent_t stage_done[2] = {nullptr, nullptr};    // the second lane has finished its chunks

  hipStream_t stream_of(const Node& n) const {
    if (n.op == LMS_OP_SWAP_OUT) return s_d2h;
    if (n.op == LMS_OP_SWAP_IN) return s_h2d;
    return s_compute;
  }
  void* ptr(int v) const {
    if (bound[v]) return bound[v];
    const Node& n = g.nodes[v];
    if (n.op == LMS_OP_SWAP_OUT) return pinned + plan.host_off[v];
    return arena + plan.block[v].off;
  }
  void* ws(int v) const { return arena + plan.wspace[v].off; }
};


namespace {

// A swap-out / swap-in of an encoded tensor through the staging buffers, chunk by chunk, on two lanes: even chunks on
// the node's own stream with staging buffer 0, odd chunks on the other side stream (idle in that phase of the step:
// swap-outs belong to the forward phase, swap-ins to the backward phase) with buffer 1.  Within a lane kernel and
// pitched copy follow each other in stream order, which is all the ordering a buffer needs (a buffer is only ever
// touched on its lane's stream, also by the next tensor); the two lanes overlap, so the copy engine of one moves a
// chunk while the other lane's kernel runs or its copy is being set up.  (One lane for all copies and one for all
// kernels, ordered by events per chunk, left the link idle for 0.15 ms between copies of 0.7 ms: a copy that waits for
// an event of another stream starts late.  Two more streams of the executor's own for the kernels were slower still,
// 108 against 90 ms on ResNet-50 at 1.5 times the unswapped batch: the device has four hardware queues, and streams
// that share one wait for each other.)  With one lane larger chunks gained (stand-alone 51.8 GB/s with 8192 slots per
// copy, 53.8 with 16384); with two lanes 8192 slots reach the same 53-54 GB/s in place as 16384 and leave the plan
// 143 MB more.
// The second lane starts after what the node's stream waited for, and the node's stream ends after the second lane's
// last operation, so the event the executor records on it afterwards covers everything.
hipError_t staged_swap_out(Exec& e, void* host, const void* src, uint64_t numel, int w, hipStream_t s) {
  const int64_t stride = (int64_t)swap_slot_stride();
  const int64_t nslots = (int64_t)((numel + swap_slot_elements() - 1) / swap_slot_elements());
  const int64_t buf_bytes = STAGE_SLOTS * stride;
  hipStream_t lane[2] = {s, s == e.s_d2h ? e.s_h2d : s};
  hipError_t err = hipEventRecord(e.stage_start[0], s);
  if (err == hipSuccess && lane[1] != s) err = hipStreamWaitEvent(lane[1], e.stage_start[0], 0);
  if (err != hipSuccess) return err;
  int j = 0;
  for (int64_t b = 0; b < nslots; b += STAGE_SLOTS, ++j) {
    const int64_t end = b + STAGE_SLOTS < nslots ? b + STAGE_SLOTS : nslots;
    const int h = j & 1;
    char* buf = e.stage_out + h * buf_bytes;
    err = swap_encode_range(host, src, numel, b, end, buf, w, 2048, lane[h]);
    if (err == hipSuccess)
      err = hipMemcpy2DAsync((char*)host + b * stride, (size_t)stride, buf, (size_t)stride, (size_t)w, (size_t)(end - b), hipMemcpyDeviceToHost, lane[h]);
    if (err != hipSuccess) return err;
  }
  if (j > 1 && lane[1] != s) {
    err = hipEventRecord(e.stage_done[0], lane[1]);
    if (err == hipSuccess) err = hipStreamWaitEvent(s, e.stage_done[0], 0);
  }
  return err;
}
hipError_t staged_swap_in(Exec& e, void* dst, const void* host, uint64_t numel, int w, hipStream_t s) {
  const int64_t stride = (int64_t)swap_slot_stride();
  const int64_t nslots = (int64_t)((numel + swap_slot_elements() - 1) / swap_slot_elements());
  const int64_t buf_bytes = STAGE_SLOTS * stride;
  hipStream_t lane[2] = {s, s == e.s_h2d ? e.s_d2h : s};
  hipError_t err = hipEventRecord(e.stage_start[1], s);
  if (err == hipSuccess && lane[1] != s) err = hipStreamWaitEvent(lane[1], e.stage_start[1], 0);
  if (err != hipSuccess) return err;
  int j = 0;
  for (int64_t b = 0; b < nslots; b += STAGE_SLOTS, ++j) {
    const int64_t end = b + STAGE_SLOTS < nslots ? b + STAGE_SLOTS : nslots;
    const int h = j & 1;
    char* buf = e.stage_in + h * buf_bytes;
    err = hipMemcpy2DAsync(buf, (size_t)stride, (const char*)host + b * stride, (size_t)stride, (size_t)w, (size_t)(end - b), hipMemcpyHostToDevice, lane[h]);
    if (err == hipSuccess) err = swap_decode_range(dst, host, numel, b, end, buf, w, 2048, lane[h]);
    if (err != hipSuccess) return err;
  }
  if (j > 1 && lane[1] != s) {
    err = hipEventRecord(e.stage_done[1], lane[1]);
    if (err == hipSuccess) err = hipStreamWaitEvent(s, e.stage_done[1], 0);
  }
  return err;
}

lms_status hip_fail(hipError_t e, const char* what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return LMS_EHIP;
}

// Nodes that touched tenant t's memory: its producer and the readers of its output.
void accessors(const Exec& e, const std::vector<std::vector<int>>& readers, int t, bool workspace_only, std::vector<int>& out) {
  out.push_back(t);
  if (!workspace_only)
    for (int r : readers[t]) out.push_back(r);
}

void build_sync(Exec& e) {
  const Graph& g = e.g;
  const int n = (int)g.nodes.size();
  std::vector<std::vector<int>> readers, outs;
  adjacency(g, readers, outs);
  e.waits.assign(n, {});
  e.poison_waits.assign(n, {});
  e.dying.assign(n, {});
  std::vector<char> need(n, 0);
  auto add_wait = [&](std::vector<int>& list, int v, int on) {
    if (g.nodes[on].is_var) return;
    if (e.stream_of(g.nodes[on]) == e.stream_of(g.nodes[v])) return;   // in-order stream
    if (std::find(list.begin(), list.end(), on) == list.end()) list.push_back(on);
    need[on] = 1;
  };
  // a node's workspace is only touched by the node itself, its output block by itself and its readers: an earlier
  // workspace tenant must not make the node wait for the readers of that operation's output (a swap-out among them
  // would hold every operation that reuses a few kilobytes of scratch for the length of the copy)
  for (const Node& v : g.nodes) {
    if (v.is_var) continue;
    for (int u : v.in) add_wait(e.waits[v.id], v.id, u);
    for (int u : v.ctrl_in) add_wait(e.waits[v.id], v.id, u);
    std::vector<int> acc;
    for (const std::vector<int>* prev : {&e.plan.prev_tenants[v.id], &e.plan.ws_prev_tenants[v.id]})
      for (int t : *prev) {
        if (t >= 0) accessors(e, readers, t, false, acc);       // an output block: its producer and its readers
        else accessors(e, readers, ~t, true, acc);              // a workspace: the operation itself
      }
    // streams run in order: per foreign stream only the accessor latest in the schedule matters
    int latest[3] = {-1, -1, -1};
    for (int a : acc) {
      const Node& na = g.nodes[a];
      if (na.is_var) continue;
      const int si = na.op == LMS_OP_SWAP_OUT ? 1 : (na.op == LMS_OP_SWAP_IN ? 2 : 0);
      if (latest[si] < 0 || e.plan.pos[a] > e.plan.pos[latest[si]]) latest[si] = a;
    }
    for (int a : latest)
      if (a >= 0) add_wait(e.waits[v.id], v.id, a);
  }
  if (!(e.flags & LMS_X_KEEP_ALL)) {
    for (const Node& v : g.nodes) {
      if (v.is_var || e.plan.block[v.id].size == 0 || e.plan.last_use[v.id] < 0 || e.plan.moved[v.id]) continue;
      const int at = e.plan.order[std::max(e.plan.last_use[v.id], e.plan.pos[v.id])];
      e.dying[at].push_back(v.id);
    }
    if (e.flags & LMS_X_POISON) {
      // the poison fill runs on the compute stream: it must wait for copies still reading the block
      for (int at = 0; at < n; ++at)
        for (int d : e.dying[at]) {
          std::vector<int> acc;
          accessors(e, readers, d, false, acc);
          for (int a : acc)
            if (e.stream_of(g.nodes[a]) != e.s_compute && !g.nodes[a].is_var) {
              if (std::find(e.poison_waits[at].begin(), e.poison_waits[at].end(), a) == e.poison_waits[at].end())
                e.poison_waits[at].push_back(a);
              need[a] = 1;
            }
        }
    }
  }
  e.ev.assign(n, nullptr);
  for (int v = 0; v < n; ++v)
    if (need[v] && hipEventCreateWithFlags(&e.ev[v], hipEventDisableTiming) != hipSuccess) { e.ev[v] = nullptr; e.events_ok = false; }
}

// fp32 check mode: the operation's activations are fp32 (the graph was built on an fp32 input batch and fp32 filters).
// Returns false if the node is not an fp32-activation operation.
bool run_node_f32(Exec& e, const Node& n, hipError_t& err) {
  const Graph& g = e.g;
  hipStream_t s = e.stream_of(n);
  auto IN = [&](int i) -> const Node& { return g.nodes[n.in[i]]; };
  auto P = [&](int i) -> void* { return e.ptr(n.in[i]); };
  void* out = e.ptr(n.id);
  const uint32_t f = n.attr.flags;
  if (n.in.empty()) return false;
  const bool act32 = n.op == LMS_OP_DOT_COLS ? IN(1).dtype == LMS_F32 : IN(0).dtype == LMS_F32;
  if (!act32) return false;
  switch (n.op) {
    case LMS_OP_CONV: {
      Epilogue ep;
      int slot = 2;
      if (f & LMS_F_AFFINE) { ep.scale = (const float*)P(slot); ep.shift = (const float*)P(slot + 1); slot += 2; }
      if (f & LMS_F_BIAS) { ep.shift = (const float*)P(slot); ++slot; }
      if (f & LMS_F_RES) ep.add = P(slot);
      ep.relu = (f & LMS_F_RELU) ? 1 : 0;
      err = check_conv(geom_of(IN(0), n, n.attr, false), 0, 0, P(0), P(1), ep, out, s);
      break;
    }
    case LMS_OP_CONV_DGRAD: case LMS_OP_TCONV_DGRAD: {
      Epilogue ep;
      int slot = 2;
      if (n.op == LMS_OP_CONV_DGRAD && (f & LMS_F_AFFINE)) ep.scale = (const float*)P(slot++);
      if (f & LMS_F_ADDEND) ep.add = P(slot++);
      if (f & LMS_F_MASK) ep.mask = P(slot++);
      const bool tc = n.op == LMS_OP_TCONV_DGRAD;
      err = check_conv(geom_of(n, IN(0), n.attr, tc), 1, tc ? 1 : 0, P(0), P(1), ep, out, s);
      break;
    }
    case LMS_OP_CONV_WGRAD: err = check_wgrad(geom_of(IN(0), IN(1), n.attr, false), 0, P(0), P(1), (float*)out, s); break;
    case LMS_OP_TCONV: {
      Epilogue ep;
      err = check_conv(geom_of(IN(0), n, n.attr, true), 0, 1, P(0), P(1), ep, out, s);
      break;
    }
    case LMS_OP_TCONV_WGRAD: err = check_wgrad(geom_of(IN(0), IN(1), n.attr, true), 1, P(0), P(1), (float*)out, s); break;
    case LMS_OP_MAXPOOL: err = check_maxpool_fwd(geom_of(IN(0), n, n.attr, false), P(0), out, s); break;
    case LMS_OP_MAXPOOL_BWD: err = check_maxpool_bwd(geom_of(n, IN(0), n.attr, false), P(0), P(1), (f & LMS_F_MASK) ? 1 : 0, out, s); break;
    case LMS_OP_GAP: {
      const Node& x = IN(0);
      err = check_gap_fwd(x.dims[0], x.numel() / x.dims[0] / x.channels(), (int)x.channels(), P(0), out, s);
      break;
    }
    case LMS_OP_GAP_BWD:
      err = check_gap_bwd(n.dims[0], n.numel() / n.dims[0] / n.channels(), (int)n.channels(), P(0), (f & LMS_F_MASK) ? P(1) : nullptr, out, s);
      break;
    case LMS_OP_CONCAT: {
      const int64_t rows = n.numel() / n.channels();
      const int ca = (int)IN(0).channels(), cb = (int)IN(1).channels();
      err = check_copy_channels(rows, P(0), ca, 0, out, ca + cb, 0, ca, nullptr, s);
      if (err == hipSuccess) err = check_copy_channels(rows, P(1), cb, 0, out, ca + cb, ca, cb, nullptr, s);
      break;
    }
    case LMS_OP_SLICE_C:
      err = check_copy_channels(n.numel() / n.channels(), P(0), (int)IN(0).channels(), n.attr.c_begin, out, (int)n.channels(), 0,
                                n.attr.c_count, (f & LMS_F_MASK) ? P(1) : nullptr, s);
      break;
    case LMS_OP_MSE: err = check_mse_loss(IN(0).numel(), P(0), P(1), (float*)out, s); break;
    case LMS_OP_MSE_GRAD: err = check_mse_grad(IN(0).numel(), P(0), P(1), (f & LMS_F_MASK) ? P(2) : nullptr, out, s); break;
    case LMS_OP_SOFTMAX_CE:
      err = check_ce_loss(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), P(0), (const int32_t*)P(1), (float*)out, s);
      break;
    case LMS_OP_SOFTMAX_CE_GRAD:
      err = check_ce_grad(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), P(0), (const int32_t*)P(1),
                          (f & LMS_F_MASK) ? P(2) : nullptr, out, s);
      break;
    case LMS_OP_GRAD_SUM: {
      const int ng = (int)n.in.size() - ((f & LMS_F_MASK) ? 1 : 0);
      const void* gp[4] = {nullptr, nullptr, nullptr, nullptr};
      for (int i = 0; i < ng; ++i) gp[i] = P(i);
      err = check_grad_sum(n.numel(), ng, gp, (f & LMS_F_MASK) ? P(ng) : nullptr, out, s);
      break;
    }
    case LMS_OP_COLSUM:
      err = check_col_reduce(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), (const float*)P(0), nullptr, (float*)out, s);
      break;
    case LMS_OP_DOT_COLS:
      err = check_col_reduce(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), (const float*)P(0), P(1), (float*)out, s);
      break;
    default: return false;      // scale_cols (fp32 in both modes) and the swap copies do not depend on the element type
  }
  e.n_kernels += 1;
  return true;
}

lms_status run_node(Exec& e, const Node& n) {
  const Graph& g = e.g;
  hipStream_t s = e.stream_of(n);
  auto IN = [&](int i) -> const Node& { return g.nodes[n.in[i]]; };
  auto P = [&](int i) -> void* { return e.ptr(n.in[i]); };
  void* out = e.ptr(n.id);
  const uint32_t f = n.attr.flags;
  hipError_t err = hipSuccess;
  if (n.op == LMS_OP_MOMENTUM) {
    // momentum * v + dp, written as dp - (-momentum) * v with the update kernel
    err = sgd_update(n.numel(), true, P(1), (const float*)P(0), -n.attr.lr, out, s);
    e.n_kernels += 1;
    if (err != hipSuccess) { set_error("executor: node %d (%s): %s", n.id, n.name.c_str(), hipGetErrorString(err)); return LMS_EHIP; }
    return LMS_OK;
  }
  if (n.op == LMS_OP_SGD) {
    err = sgd_update(n.numel(), n.dtype == LMS_F32, P(0), (const float*)P(1), n.attr.lr, out, s);
    e.n_kernels += 1;
    if (err != hipSuccess) { set_error("executor: node %d (%s): %s", n.id, n.name.c_str(), hipGetErrorString(err)); return LMS_EHIP; }
    return LMS_OK;
  }
  if (run_node_f32(e, n, err)) {
    if (err != hipSuccess) {
      set_error("executor (fp32 check): node %d (%s, op %d): %s", n.id, n.name.c_str(), n.op, hipGetErrorString(err));
      return LMS_EHIP;
    }
    return LMS_OK;
  }
  switch (n.op) {
    case LMS_OP_CONV: {
      Epilogue ep;
      int slot = 2;
      if (f & LMS_F_AFFINE) { ep.scale = (const float*)P(slot); ep.shift = (const float*)P(slot + 1); slot += 2; }
      if (f & LMS_F_BIAS) { ep.shift = (const float*)P(slot); ++slot; }
      if (f & LMS_F_RES) ep.add = P(slot);
      ep.relu = (f & LMS_F_RELU) ? 1 : 0;
      err = conv_fwd(geom_of(IN(0), n, n.attr, false), P(0), P(1), ep, out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    }
    case LMS_OP_CONV_DGRAD: case LMS_OP_TCONV_DGRAD: {
      Epilogue ep;
      int slot = 2;
      if (n.op == LMS_OP_CONV_DGRAD && (f & LMS_F_AFFINE)) ep.scale = (const float*)P(slot++);
      if (f & LMS_F_ADDEND) ep.add = P(slot++);
      if (f & LMS_F_MASK) ep.mask = P(slot++);
      if (n.op == LMS_OP_CONV_DGRAD) err = conv_dgrad(geom_of(n, IN(0), n.attr, false), P(0), P(1), ep, out, e.ws(n.id), s);
      else err = tconv_dgrad(geom_of(n, IN(0), n.attr, true), P(0), P(1), ep, out, s);
      e.n_kernels += 1;
      break;
    }
    case LMS_OP_CONV_WGRAD: {
      // the column sums of the same dy (a COLSUM node bound to caller memory) come out of this pass
      const int c = wgrad_side_colsum(g, n.id);
      err = conv_wgrad(geom_of(IN(0), IN(1), n.attr, false), P(0), P(1), (float*)out, e.ws(n.id), s, c >= 0 ? (float*)e.ptr(c) : nullptr);
      e.n_kernels += c >= 0 ? 3 : 2;
      break;
    }
    case LMS_OP_TCONV:
      err = tconv_fwd(geom_of(IN(0), n, n.attr, true), P(0), P(1), out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    case LMS_OP_TCONV_WGRAD:
      err = tconv_wgrad(geom_of(IN(0), IN(1), n.attr, true), P(0), P(1), (float*)out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    case LMS_OP_MAXPOOL: {
      ConvGeom pg = geom_of(IN(0), n, n.attr, false);
      err = maxpool_fwd(pg, P(0), out, s);
      e.n_kernels += 1;
      break;
    }
    case LMS_OP_MAXPOOL_BWD: {
      ConvGeom pg = geom_of(n, IN(0), n.attr, false);
      err = maxpool_bwd(pg, P(0), P(1), (f & LMS_F_MASK) ? 1 : 0, out, s);
      e.n_kernels += 1;
      break;
    }
    case LMS_OP_GAP: {
      const Node& x = IN(0);
      err = gap_fwd(x.dims[0], x.numel() / x.dims[0] / x.channels(), (int)x.channels(), P(0), out, s);
      e.n_kernels += 1;
      break;
    }
    case LMS_OP_GAP_BWD:
      err = gap_bwd(n.dims[0], n.numel() / n.dims[0] / n.channels(), (int)n.channels(), P(0), (f & LMS_F_MASK) ? P(1) : nullptr, out, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_CONCAT: {
      const int64_t rows = n.numel() / n.channels();
      const int ca = (int)IN(0).channels(), cb = (int)IN(1).channels();
      err = copy_channels(rows, P(0), ca, 0, out, ca + cb, 0, ca, nullptr, s);
      if (err == hipSuccess) err = copy_channels(rows, P(1), cb, 0, out, ca + cb, ca, cb, nullptr, s);
      e.n_kernels += 2;
      break;
    }
    case LMS_OP_SLICE_C:
      err = copy_channels(n.numel() / n.channels(), P(0), (int)IN(0).channels(), n.attr.c_begin, out, (int)n.channels(), 0,
                          n.attr.c_count, (f & LMS_F_MASK) ? P(1) : nullptr, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_MSE:
      err = mse_loss(IN(0).numel(), P(0), P(1), (float*)out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    case LMS_OP_MSE_GRAD:
      err = mse_grad(IN(0).numel(), P(0), P(1), (f & LMS_F_MASK) ? P(2) : nullptr, out, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_SOFTMAX_CE:
      err = softmax_ce_loss(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), P(0), (const int32_t*)P(1), (float*)out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    case LMS_OP_SOFTMAX_CE_GRAD:
      err = softmax_ce_grad(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), P(0), (const int32_t*)P(1),
                            (f & LMS_F_MASK) ? P(2) : nullptr, out, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_GRAD_SUM: {
      const int ng = (int)n.in.size() - ((f & LMS_F_MASK) ? 1 : 0);
      const void* gp[4] = {nullptr, nullptr, nullptr, nullptr};
      for (int i = 0; i < ng; ++i) gp[i] = P(i);
      err = grad_sum(n.numel(), ng, gp, (f & LMS_F_MASK) ? P(ng) : nullptr, out, s);
      e.n_kernels += 1;
      break;
    }
    case LMS_OP_COLSUM:
      if (colsum_host_wgrad(g, n.id) >= 0) break;          // written by the weight-gradient node earlier in the step
      err = colsum(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), P(0), (float*)out, e.ws(n.id), s);
      e.n_kernels += 2;
      break;
    case LMS_OP_SCALE_COLS:
      err = scale_cols(n.numel() / n.channels(), (int)n.channels(), (const float*)P(0), (const float*)P(1), (float*)out, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_DOT_COLS:
      err = dot_cols(IN(0).numel() / IN(0).channels(), (int)IN(0).channels(), (const float*)P(0), P(1), (float*)out, s);
      e.n_kernels += 1;
      break;
    case LMS_OP_SWAP_OUT:
      if (e.flags & LMS_X_DMA_COPY) err = hipMemcpyAsync(out, P(0), n.bytes(), hipMemcpyDeviceToHost, s);
      // no trailer kernel on the swap stream: the step's statistics count the bytes on the host afterwards
      else if (e.encodes(n) && e.stage_out && e.stage_w[n.id] > 0) err = staged_swap_out(e, out, P(0), (uint64_t)n.numel(), e.stage_w[n.id], s);
      else if (e.encodes(n)) err = swap_encode(out, P(0), (uint64_t)n.numel(), e.encode_blocks, s, false);
      else err = swap_copy(out, P(0), n.bytes(), e.copy_blocks, s);
      if (!e.encodes(n)) e.bytes_d2h += n.bytes();      // encoded copies are counted from the slot headers after the step
      e.n_copies += 1;
      break;
    case LMS_OP_SWAP_IN:
      if (e.flags & LMS_X_DMA_COPY) err = hipMemcpyAsync(out, P(0), n.bytes(), hipMemcpyHostToDevice, s);
      else if (e.encodes(n) && e.stage_in && e.stage_w[n.in[0]] > 0) err = staged_swap_in(e, out, P(0), (uint64_t)n.numel(), e.stage_w[n.in[0]], s);
      else if (e.encodes(n)) err = swap_decode(out, P(0), (uint64_t)n.numel(), e.decode_blocks, s);
      else err = swap_copy(out, P(0), n.bytes(), e.copy_blocks, s);
      if (!e.encodes(n)) e.bytes_h2d += n.bytes();
      e.n_copies += 1;
      break;
    default:
      set_error("executor: op %d (%s) not implemented", n.op, n.name.c_str());
      return LMS_EINVAL;
  }
  if (err != hipSuccess) {
    set_error("executor: node %d (%s, op %d): %s", n.id, n.name.c_str(), n.op, hipGetErrorString(err));
    return LMS_EHIP;
  }
  return LMS_OK;
}

}  // namespace

lms_status exec_destroy(Exec* e);

lms_status exec_create(const Graph& g, void* arena, uint64_t arena_bytes, void* pinned, uint64_t pinned_bytes,
                       void* sc, void* sd, void* sh, uint32_t flags, Exec** out) {
  if (!out || (!arena && arena_bytes)) { set_error("lms_exec_create: bad argument"); return LMS_EINVAL; }
  if (((uintptr_t)arena & 255u) != 0) { set_error("lms_exec_create: arena must be 256-byte aligned"); return LMS_EINVAL; }
  Exec* e = new Exec();
  e->g = g;
  const bool encode = (flags & LMS_X_ENCODE_SWAPS) && !(flags & LMS_X_DMA_COPY);
  const bool staged = encode && (flags & LMS_X_STAGED_SWAPS);
  uint64_t plan_bytes = arena_bytes;
  if (staged) {
    // the staging buffers take the end of the arena
    if (arena_bytes < swap_staging_bytes() + 256) {
      delete e;
      set_error("lms_exec_create: LMS_X_STAGED_SWAPS needs %llu bytes of the arena for its staging buffers, the arena has %llu",
                (unsigned long long)swap_staging_bytes(), (unsigned long long)arena_bytes);
      return LMS_EOOM_DEVICE;
    }
    plan_bytes = (arena_bytes - swap_staging_bytes()) & ~(uint64_t)255;
  }
  plan_memory(e->g, plan_bytes ? plan_bytes : 1, (flags & LMS_X_KEEP_ALL) != 0, nullptr, e->plan, encode);
  if ((int)e->plan.order.size() != (int)g.nodes.size()) { delete e; set_error("lms_exec_create: graph has a cycle"); return LMS_ECYCLE; }
  if (!e->plan.fits) {
    PlanResult need;
    plan_memory(e->g, 0, (flags & LMS_X_KEEP_ALL) != 0, nullptr, need);
    set_error("lms_exec_create: arena of %llu bytes%s is too small, the graph as it is needs %llu",
              (unsigned long long)plan_bytes, staged ? " (without the staging buffers)" : "", (unsigned long long)need.arena_needed);
    delete e;
    return LMS_EOOM_DEVICE;
  }
  if (e->plan.pinned_needed > pinned_bytes) {
    set_error("lms_exec_create: pinned pool of %llu bytes is too small, swapped tensors need %llu",
              (unsigned long long)pinned_bytes, (unsigned long long)e->plan.pinned_needed);
    delete e;
    return LMS_EOOM_HOST;
  }
  e->arena = (char*)arena;
  e->arena_bytes = arena_bytes;
  e->pinned = (char*)pinned;
  e->pinned_bytes = pinned_bytes;
  e->flags = flags;
  e->s_compute = (hipStream_t)sc;
  e->s_d2h = (flags & LMS_X_NO_OVERLAP) ? (hipStream_t)sc : (hipStream_t)sd;
  e->s_h2d = (flags & LMS_X_NO_OVERLAP) ? (hipStream_t)sc : (hipStream_t)sh;
  e->bound.assign(g.nodes.size(), nullptr);
  e->stage_w.assign(g.nodes.size(), 0);
  if (staged) {
    e->stage_out = e->arena + plan_bytes;
    e->stage_in = e->stage_out + swap_staging_bytes() / 2;
    auto make = [&](hipEvent_t& ev) { if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { ev = nullptr; e->events_ok = false; } };
    for (int d = 0; d < 2; ++d) {
      make(e->stage_start[d]);
      make(e->stage_done[d]);
    }
  }
  if (const char* cb = getenv("LMS_COPY_BLOCKS")) { const int v = atoi(cb); if (v > 0 && v <= 4096) e->copy_blocks = v; }
  if (const char* cb = getenv("LMS_ENCODE_BLOCKS")) { const int v = atoi(cb); if (v > 0 && v <= 4096) e->encode_blocks = v; }
  if (const char* cb = getenv("LMS_DECODE_BLOCKS")) { const int v = atoi(cb); if (v > 0 && v <= 4096) e->decode_blocks = v; }
  build_sync(*e);
  if (flags & LMS_X_TIMING) {
    const int n = (int)g.nodes.size();
    e->wait_span.assign(n, Exec::WaitSpan());
    e->copy_begin.assign(n, nullptr);
    e->copy_end.assign(n, nullptr);
    auto make = [&](hipEvent_t& ev) { if (hipEventCreate(&ev) != hipSuccess) { ev = nullptr; e->events_ok = false; } };
    make(e->step_begin);
    make(e->step_end);
    for (const Node& v : e->g.nodes) {
      if (v.is_var) continue;
      hipStream_t s = e->stream_of(v);
      if (s == e->s_compute) {
        Exec::WaitSpan& w = e->wait_span[v.id];
        for (int on : e->waits[v.id]) {
          hipStream_t so = e->stream_of(e->g.nodes[on]);
          if (so == e->s_h2d && so != e->s_compute) w.on_h2d = true;
          else if (so == e->s_d2h && so != e->s_compute) w.on_d2h = true;
        }
        if (w.on_h2d || w.on_d2h) { make(w.before); make(w.after); }
      } else {
        make(e->copy_begin[v.id]);
        make(e->copy_end[v.id]);
      }
    }
  }
  if (hipEventCreateWithFlags(&e->join_d2h, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&e->join_h2d, hipEventDisableTiming) != hipSuccess || !e->events_ok) {
    exec_destroy(e);
    set_error("lms_exec_create: hipEventCreate failed");
    return LMS_EHIP;
  }
  *out = e;
  return LMS_OK;
}

lms_status pinned_alloc(uint64_t bytes, void** out) {
  void* p = nullptr;
  const hipError_t err = hipHostMalloc(&p, bytes, hipHostMallocDefault);
  if (err != hipSuccess || !p) {
    (void)hipGetLastError();      // the failed allocation must not be reported by the next call
    set_error("lms_pinned_alloc: hipHostMalloc of %llu bytes failed: %s", (unsigned long long)bytes, hipGetErrorString(err));
    return err == hipErrorOutOfMemory ? LMS_EOOM_HOST : LMS_EHIP;
  }
  *out = p;
  return LMS_OK;
}

lms_status pinned_free(void* p) {
  if (!p) return LMS_OK;
  hipError_t err = hipDeviceSynchronize();
  if (err == hipSuccess) err = hipHostFree(p);
  return err == hipSuccess ? LMS_OK : hip_fail(err, "lms_pinned_free");
}

lms_status exec_destroy(Exec* e) {
  if (!e) return LMS_OK;
  for (int d = 0; d < 2; ++d) {
    if (e->stage_start[d]) (void)hipEventDestroy(e->stage_start[d]);
    if (e->stage_done[d]) (void)hipEventDestroy(e->stage_done[d]);
  }
  for (hipEvent_t ev : e->ev)
    if (ev) (void)hipEventDestroy(ev);
  for (auto& w : e->wait_span) {
    if (w.before) (void)hipEventDestroy(w.before);
    if (w.after) (void)hipEventDestroy(w.after);
  }
  for (hipEvent_t ev : e->copy_begin)
    if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : e->copy_end)
    if (ev) (void)hipEventDestroy(ev);
  if (e->step_begin) (void)hipEventDestroy(e->step_begin);
  if (e->step_end) (void)hipEventDestroy(e->step_end);
  if (e->join_d2h) (void)hipEventDestroy(e->join_d2h);
  if (e->join_h2d) (void)hipEventDestroy(e->join_h2d);
  delete e;
  return LMS_OK;
}

lms_status exec_set_swap_grid(Exec* e, int encode_wgs, int decode_wgs) {
  if (encode_wgs < 0 || encode_wgs > 4096 || decode_wgs < 0 || decode_wgs > 4096) {
    set_error("lms_exec_set_swap_grid: %d / %d work-groups, 0 to 4096 each", encode_wgs, decode_wgs);
    return LMS_EINVAL;
  }
  if (encode_wgs) e->encode_blocks = encode_wgs;
  if (decode_wgs) e->decode_blocks = decode_wgs;
  return LMS_OK;
}

lms_status exec_bind(Exec* e, int node, void* p) {
  if (!e || node < 0 || node >= (int)e->g.nodes.size() || !p) { set_error("lms_exec_bind: bad argument"); return LMS_EINVAL; }
  const int op = e->g.nodes[node].op;
  if (op == LMS_OP_SWAP_OUT || op == LMS_OP_SWAP_IN) { set_error("lms_exec_bind: swap operations cannot be bound"); return LMS_EINVAL; }
  e->bound[node] = p;
  return LMS_OK;
}

lms_status exec_tensor_ptr(Exec* e, int node, void** p) {
  if (!e || !p || node < 0 || node >= (int)e->g.nodes.size()) { set_error("lms_exec_tensor_ptr: bad argument"); return LMS_EINVAL; }
  if (e->g.nodes[node].is_var && !e->bound[node]) { set_error("lms_exec_tensor_ptr: variable not bound"); return LMS_EINVAL; }
  *p = e->ptr(node);
  return LMS_OK;
}

namespace {

// An update may wait for the others of its step if it touches caller memory only (parameter, gradient and result bound
// with lms_exec_bind: no arena block whose reuse the plan has ordered), and nothing waits for it across streams.
bool can_defer_update(const Exec& e, const Node& n) {
  if (n.op != LMS_OP_SGD || n.in.size() != 2 || n.numel() <= 0 || n.numel() > (1ll << 38)) return false;
  if (!e.bound[n.id] || !e.bound[n.in[0]] || !e.bound[n.in[1]]) return false;
  if (!e.waits[n.id].empty() || e.ev[n.id] || !n.ctrl_in.empty()) return false;
  if ((int)e.dying.size() > n.id && !e.dying[n.id].empty()) return false;
  return e.stream_of(n) == e.s_compute;
}

lms_status flush_updates(Exec& e) {
  size_t at = 0;
  while (at < e.pending.size()) {
    SgdBatch b;
    b.count = 0;
    b.f32_mask = 0;
    b.first[0] = 0;
    while (at < e.pending.size() && b.count < SGD_BATCH) {
      const Node& n = e.g.nodes[e.pending[at]];
      const int blocks = sgd_batch_blocks(n.numel());
      if (b.count > 0 && (long long)b.first[b.count] + blocks > 0x3fffffffLL) break;
      const int t = b.count++;
      b.p[t] = e.ptr(n.in[0]);
      b.g[t] = (const float*)e.ptr(n.in[1]);
      b.out[t] = e.ptr(n.id);
      b.n[t] = n.numel();
      b.lr[t] = n.attr.lr;
      if (n.dtype == LMS_F32) b.f32_mask |= 1ull << t;
      b.first[t + 1] = b.first[t] + blocks;
      ++at;
    }
    const hipError_t err = sgd_update_batch(b, e.s_compute);
    e.n_kernels += 1;
    if (err != hipSuccess) { set_error("executor: batched update: %s", hipGetErrorString(err)); return LMS_EHIP; }
  }
  for (int v : e.pending) { e.pend_mark[v] = 0; e.pend_mark[e.g.nodes[v].in[0]] = 0; }
  e.pending.clear();
  return LMS_OK;
}

}  // namespace

lms_status exec_step(Exec* e, float* loss_out, lms_step_stats* stats) {
  if (!e) { set_error("lms_exec_step: null executor"); return LMS_EINVAL; }
  const Graph& g = e->g;
  int loss_node = -1;
  for (const Node& n : g.nodes) {
    if (n.is_var && !e->bound[n.id]) { set_error("lms_exec_step: variable %s is not bound", n.name.c_str()); return LMS_EINVAL; }
    if (n.external && !e->bound[n.id]) { set_error("lms_exec_step: %s was declared external and is not bound", n.name.c_str()); return LMS_EINVAL; }
    if (n.op == LMS_OP_MSE || n.op == LMS_OP_SOFTMAX_CE) loss_node = n.id;
  }
  e->bytes_d2h = e->bytes_h2d = 0;
  e->n_kernels = e->n_copies = 0;
  e->pending.clear();
  e->pend_mark.assign(g.nodes.size(), 0);
  auto t0 = std::chrono::steady_clock::now();
  const bool side_streams = e->s_d2h != e->s_compute || e->s_h2d != e->s_compute;
  static const bool host_trace = getenv("LMS_HOST_TRACE") != nullptr;   // prints host-side issue times of slow nodes
  const bool timing = (e->flags & LMS_X_TIMING) != 0;
  if (timing) (void)hipEventRecord(e->step_begin, e->s_compute);
  for (int v : e->plan.order) {
    const Node& n = g.nodes[v];
    if (n.is_var) continue;
    if (can_defer_update(*e, n)) {
      e->pending.push_back(v);
      e->pend_mark[v] = e->pend_mark[n.in[0]] = 1;
      continue;
    }
    if (!e->pending.empty()) {
      // an operation that reads an updated variable (it was created after the update) or the update itself
      bool touches = false;
      for (int u : n.in) touches = touches || e->pend_mark[u];
      for (int u : n.ctrl_in) touches = touches || e->pend_mark[u];
      if (touches) {
        lms_status st = flush_updates(*e);
        if (st != LMS_OK) return st;
      }
    }
    hipStream_t s = e->stream_of(n);
    auto h0 = std::chrono::steady_clock::now();
    const bool span = timing && s == e->s_compute && e->wait_span[v].before;
    if (span) (void)hipEventRecord(e->wait_span[v].before, s);
    for (int w : e->waits[v]) {
      hipError_t err = hipStreamWaitEvent(s, e->ev[w], 0);
      if (err != hipSuccess) return hip_fail(err, "hipStreamWaitEvent");
    }
    if (span) (void)hipEventRecord(e->wait_span[v].after, s);
    const bool copy_span = timing && s != e->s_compute && e->copy_begin[v];
    if (copy_span) (void)hipEventRecord(e->copy_begin[v], s);
    if ((e->flags & LMS_X_POISON) && n.op == LMS_OP_SWAP_IN && s != e->s_compute) {
      // poison fills are extra writers on the compute stream: a copy into a released block waits for all of them
      (void)hipEventRecord(e->join_h2d, e->s_compute);
      (void)hipStreamWaitEvent(s, e->join_h2d, 0);
    }
    lms_status st = run_node(*e, n);
    if (st != LMS_OK) return st;
    if (copy_span) (void)hipEventRecord(e->copy_end[v], s);
    if (e->ev[v] && s != e->s_compute) {
      hipError_t err = hipEventRecord(e->ev[v], s);
      if (err != hipSuccess) return hip_fail(err, "hipEventRecord");
    }
    if ((e->flags & LMS_X_POISON) && !e->dying[v].empty()) {
      for (int w : e->poison_waits[v]) (void)hipStreamWaitEvent(e->s_compute, e->ev[w], 0);
      for (int d : e->dying[v]) {
        if (e->bound[d]) continue;
        (void)fill16(e->arena + e->plan.block[d].off, e->g.nodes[d].bytes(), 0x7fc0, e->s_compute);
      }
    }
    // a compute node's event also covers the poison fills issued after it, which write the released blocks
    if (e->ev[v] && s == e->s_compute) {
      hipError_t err = hipEventRecord(e->ev[v], s);
      if (err != hipSuccess) return hip_fail(err, "hipEventRecord");
    }
    if (host_trace) {
      const float us = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - h0).count();
      const float at = std::chrono::duration<float, std::micro>(h0 - t0).count();
      if (us > 100.f) fprintf(stderr, "[lms host] +%9.1f us  %-40s issue took %9.1f us (%zu waits)\n", at, n.name.c_str(), us, e->waits[v].size());
    }
  }
  if (!e->pending.empty()) {
    lms_status st = flush_updates(*e);
    if (st != LMS_OK) return st;
  }
  if (side_streams) {   // join: whoever uses the compute stream next sees every copy finished
    if (e->s_d2h != e->s_compute) { (void)hipEventRecord(e->join_d2h, e->s_d2h); (void)hipStreamWaitEvent(e->s_compute, e->join_d2h, 0); }
    if (e->s_h2d != e->s_compute) { (void)hipEventRecord(e->join_h2d, e->s_h2d); (void)hipStreamWaitEvent(e->s_compute, e->join_h2d, 0); }
  }
  if (timing) (void)hipEventRecord(e->step_end, e->s_compute);
  float ms = 0.f;
  if (loss_out) {
    hipError_t err = hipStreamSynchronize(e->s_compute);
    if (err != hipSuccess) return hip_fail(err, "hipStreamSynchronize");
    ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *loss_out = 0.f;
    if (loss_node >= 0) {
      err = hipMemcpy(loss_out, e->ptr(loss_node), sizeof(float), hipMemcpyDeviceToHost);
      if (err != hipSuccess) return hip_fail(err, "hipMemcpy(loss)");
    }
  }
  if (loss_out && (e->flags & LMS_X_ENCODE_SWAPS)) {
    // the step has finished: the slot counts in the host pool say how many bytes each encoded copy moved, and give
    // the staged width of the next step (swap-ins first: they ran with the width their swap-out node still holds)
    for (int pass = 0; pass < 2; ++pass)
      for (const Node& n : e->g.nodes) {
        if (n.op != (pass == 0 ? LMS_OP_SWAP_IN : LMS_OP_SWAP_OUT) || !e->encodes(n)) continue;
        const int so = n.op == LMS_OP_SWAP_OUT ? n.id : n.in[0];
        int w_next = 0;
        uint64_t moved = 0;
        (void)swap_slot_statistics(e->pinned + e->plan.host_off[so], (uint64_t)n.numel(), e->stage_w[so], &w_next, &moved);
        if (n.op == LMS_OP_SWAP_OUT) { e->bytes_d2h += moved; if (e->stage_out) e->stage_w[so] = w_next; }
        else e->bytes_h2d += moved;
      }
    e->last_enc_d2h = e->bytes_d2h;
    e->last_enc_h2d = e->bytes_h2d;
  } else if (e->flags & LMS_X_ENCODE_SWAPS) {
    // not finished yet: the sizes of this step's encoded copies are not known; report the latest finished step's
    e->bytes_d2h += e->last_enc_d2h;
    e->bytes_h2d += e->last_enc_h2d;
  }
  if (stats) {
    stats->ms = ms;
    stats->stall_h2d_ms = stats->stall_d2h_ms = stats->busy_d2h_ms = stats->busy_h2d_ms = stats->device_ms = 0.f;
    if (timing && loss_out) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, e->step_begin, e->step_end) == hipSuccess) stats->device_ms = t;
      for (const Node& n : e->g.nodes) {
        if (n.is_var) continue;
        const Exec::WaitSpan& w = e->wait_span[n.id];
        if (w.before && hipEventElapsedTime(&t, w.before, w.after) == hipSuccess) {
          // a node that waits for both directions is booked on the swap-in side: its data must arrive, a released
          // block is usually free long before
          if (w.on_h2d) stats->stall_h2d_ms += t;
          else stats->stall_d2h_ms += t;
        }
        if (e->copy_begin[n.id] && hipEventElapsedTime(&t, e->copy_begin[n.id], e->copy_end[n.id]) == hipSuccess) {
          if (n.op == LMS_OP_SWAP_OUT) stats->busy_d2h_ms += t;
          else stats->busy_h2d_ms += t;
        }
      }
    }
    stats->bytes_d2h = e->bytes_d2h;
    stats->bytes_h2d = e->bytes_h2d;
    stats->arena_bytes_used = e->plan.arena_needed;
    stats->pinned_bytes_used = e->plan.pinned_needed;
    stats->n_kernels = e->n_kernels;
    stats->n_copies = e->n_copies;
  }
  return LMS_OK;
}

}  // namespace lms

// ---- stand-alone kernel entry points ----------------------------------------------------------
namespace lms {

static bool desc_geom(const lms_conv_desc* d, ConvGeom& g) {
  if (d->ndim_sp < 2 || d->ndim_sp > 3 || d->n <= 0 || d->c <= 0 || d->k <= 0 || d->stride < 1 || d->pad < 0) return false;
  g = ConvGeom();
  g.n = d->n;
  g.c = d->c;
  g.k = d->k;
  for (int i = 0; i < d->ndim_sp; ++i) {
    const int ax = 3 - d->ndim_sp + i;
    if (d->in_sp[i] <= 0 || d->filt[i] <= 0) return false;
    g.in_sp[ax] = (int)d->in_sp[i];
    g.filt[ax] = d->filt[i];
    g.stride[ax] = d->stride;
    g.pad[ax] = d->pad;
    const int64_t o = (d->in_sp[i] + 2 * d->pad - d->filt[i]) / d->stride + 1;
    if (d->in_sp[i] + 2 * d->pad < d->filt[i] || o <= 0) return false;
    g.out_sp[ax] = (int)o;
  }
  return true;
}

// geometry of a stand-alone descriptor for entry points defined in other files
lms_status desc_to_geom(const lms_conv_desc* d, ConvGeom& g) { return desc_geom(d, g) ? LMS_OK : LMS_EINVAL; }

lms_status standalone_ws(const lms_conv_desc* d, int which, uint64_t* bytes) {
  ConvGeom g;
  if (!desc_geom(d, g)) { set_error("lms_conv_workspace_bytes: bad descriptor"); return LMS_EINVAL; }
  if (which == LMS_CONV_FWD) *bytes = conv_fwd_ws(g);
  else if (which == LMS_CONV_DGRAD_K) *bytes = conv_dgrad_ws(g, true);
  else if (which == LMS_CONV_WGRAD_K) *bytes = conv_wgrad_ws(g);
  else if (which == LMS_CONV_WGRAD_BIAS_K) *bytes = conv_wgrad_ws(g, true);
  else { set_error("lms_conv_workspace_bytes: unknown kernel %d", which); return LMS_EINVAL; }
  return LMS_OK;
}

lms_status standalone_conv(const lms_conv_desc* d, int which, const void* a, const void* b, const float* scale,
                           const float* shift, const void* add, const void* mask, void* out, void* ws, void* stream) {
  ConvGeom g;
  if (!desc_geom(d, g)) { set_error("lms_conv: bad descriptor"); return LMS_EINVAL; }
  uint64_t need = 0;
  standalone_ws(d, which, &need);
  if (which == LMS_CONV_DGRAD_K && !scale) need = conv_dgrad_ws(g, false);
  if (need && !ws) { set_error("lms_conv: workspace of %llu bytes required", (unsigned long long)need); return LMS_EINVAL; }
  Epilogue ep;
  ep.scale = scale;
  ep.shift = shift;
  ep.add = add;
  ep.mask = mask;
  ep.relu = (which == LMS_CONV_FWD && (d->flags & LMS_F_RELU)) ? 1 : 0;
  hipError_t err;
  if (which == LMS_CONV_FWD) err = conv_fwd(g, a, b, ep, out, ws, (hipStream_t)stream);
  else if (which == LMS_CONV_DGRAD_K) err = conv_dgrad(g, a, b, ep, out, ws, (hipStream_t)stream);
  else if (which == LMS_CONV_WGRAD_K) err = conv_wgrad(g, a, b, (float*)out, ws, (hipStream_t)stream);
  else err = conv_wgrad(g, a, b, (float*)out, ws, (hipStream_t)stream, const_cast<float*>(shift));    // shift slot: the bias gradient
  if (err != hipSuccess) { set_error("lms_conv: %s", hipGetErrorString(err)); return LMS_EHIP; }
  return LMS_OK;
}

}  // namespace lms

namespace lms {
lms_status swap_codec(void* dst, const void* src, uint64_t numel, bool encode, void* stream) {
  int eb = 512, db = 512;
  if (const char* cb = getenv("LMS_ENCODE_BLOCKS")) { const int v = atoi(cb); if (v > 0 && v <= 4096) eb = v; }
  if (const char* cb = getenv("LMS_DECODE_BLOCKS")) { const int v = atoi(cb); if (v > 0 && v <= 4096) db = v; }
  const hipError_t err = encode ? swap_encode(dst, src, numel, eb, (hipStream_t)stream) : swap_decode(dst, src, numel, db, (hipStream_t)stream);
  if (err != hipSuccess) { set_error("lms_swap_%s: %s", encode ? "encode" : "decode", hipGetErrorString(err)); return LMS_EHIP; }
  return LMS_OK;
}

lms_status swap_codec_staged(void* dst, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end, void* stage, int w, bool encode,
                             void* stream) {
  const hipError_t err = encode ? swap_encode_range(dst, src, numel, slot_begin, slot_end, stage, w, 2048, (hipStream_t)stream)
                                : swap_decode_range(dst, src, numel, slot_begin, slot_end, stage, w, 2048, (hipStream_t)stream);
  if (err == hipErrorInvalidValue) { set_error("lms_swap_%s_staged: slot range or width out of range", encode ? "encode" : "decode"); return LMS_EINVAL; }
  if (err != hipSuccess) { set_error("lms_swap_%s_staged: %s", encode ? "encode" : "decode", hipGetErrorString(err)); return LMS_EHIP; }
  return LMS_OK;
}

lms_status mfma_probe(uint32_t iters, bool random_operands, uint64_t* flops, void* stream) {
  if (flops) *flops = mfma_probe_flops(iters);
  hipError_t err = launch_mfma_probe(iters, random_operands ? 1 : 0, (hipStream_t)stream);
  if (err != hipSuccess) { set_error("lms_mfma_probe: %s", hipGetErrorString(err)); return LMS_EHIP; }
  return LMS_OK;
}

lms_status device_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  hipError_t err = swap_copy(dst, src, bytes, 4096, (hipStream_t)stream);
  if (err != hipSuccess) { set_error("lms_device_copy: %s", hipGetErrorString(err)); return LMS_EHIP; }
  return LMS_OK;
}
}  // namespace lms
