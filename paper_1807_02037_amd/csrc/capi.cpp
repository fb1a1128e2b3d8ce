// extern "C" surface of the library: argument checking and marshalling only.
#include <cstdint>
#include <cstring>
#include <new>

#include "graph.hpp"

struct lms_graph { lms::Graph g; };

namespace lms {
struct Exec;
lms_status exec_create(const Graph& g, void* arena, uint64_t arena_bytes, void* pinned, uint64_t pinned_bytes,
                       void* sc, void* sd, void* sh, uint32_t flags, Exec** out);
lms_status exec_destroy(Exec* e);
lms_status pinned_alloc(uint64_t bytes, void** out);
lms_status pinned_free(void* p);
lms_status exec_bind(Exec* e, int node, void* p);
lms_status exec_set_swap_grid(Exec* e, int encode_wgs, int decode_wgs);
lms_status exec_step(Exec* e, float* loss_out, lms_step_stats* stats);
lms_status exec_tensor_ptr(Exec* e, int node, void** p);
lms_status standalone_conv(const lms_conv_desc* d, int which, const void* a, const void* b, const float* scale,
                           const float* shift, const void* add, const void* mask, void* out, void* ws, void* stream);
lms_status standalone_ws(const lms_conv_desc* d, int which, uint64_t* bytes);
lms_status device_copy(void* dst, const void* src, uint64_t bytes, void* stream);
lms_status mfma_probe(uint32_t iters, bool random_operands, uint64_t* flops, void* stream);
lms_status swap_codec(void* dst, const void* src, uint64_t numel, bool encode, void* stream);
uint64_t swap_staging_bytes();
lms_status swap_codec_staged(void* dst, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end, void* stage, int w, bool encode,
                             void* stream);
uint64_t swap_encoded_bytes(uint64_t numel);
uint64_t swap_encoded_moved_bytes(const void* host, uint64_t numel);
}  // namespace lms

using lms::set_error;

#define NEED(cond, msg)        \
  do {                         \
    if (!(cond)) {             \
      set_error("%s", msg);    \
      return LMS_EINVAL;       \
    }                          \
  } while (0)

extern "C" {

const char* lms_last_error(void) { return lms::get_error(); }
const char* lms_version(void) { return "lms-mi355x 0.1 (gfx950)"; }

lms_status lms_graph_create(lms_graph** out) {
  NEED(out, "lms_graph_create: null output");
  *out = new (std::nothrow) lms_graph();
  NEED(*out, "lms_graph_create: out of host memory");
  return LMS_OK;
}
lms_status lms_graph_destroy(lms_graph* g) { delete g; return LMS_OK; }
lms_status lms_graph_clone(const lms_graph* g, lms_graph** out) {
  NEED(g && out, "lms_graph_clone: null argument");
  *out = new (std::nothrow) lms_graph(*g);
  NEED(*out, "lms_graph_clone: out of host memory");
  return LMS_OK;
}
lms_status lms_add_variable(lms_graph* g, const char* name, lms_dtype dtype, int32_t ndim, const int64_t* dims,
                            lms_var_kind kind, int32_t* node_out) {
  NEED(g, "lms_add_variable: null graph");
  return lms::add_variable(g->g, name, dtype, ndim, dims, kind, node_out);
}
lms_status lms_add_op(lms_graph* g, const char* name, lms_op op, const lms_attr* attr, int32_t n_in, const int32_t* inputs,
                      lms_phase phase, int32_t* node_out) {
  NEED(g, "lms_add_op: null graph");
  NEED(op != LMS_OP_VARIABLE, "lms_add_op: use lms_add_variable for variables");
  return lms::add_op(g->g, name, op, attr, n_in, inputs, phase, node_out);
}
lms_status lms_add_update_edge(lms_graph* g, int32_t from, int32_t var) {
  NEED(g, "lms_add_update_edge: null graph");
  const int n = (int)g->g.nodes.size();
  NEED(from >= 0 && from < n && var >= 0 && var < n, "lms_add_update_edge: unknown node");
  NEED(g->g.nodes[var].is_var, "lms_add_update_edge: target must be a variable");
  g->g.updates.emplace_back(from, var);
  return LMS_OK;
}
lms_status lms_add_control_edge(lms_graph* g, int32_t from, int32_t to) {
  NEED(g, "lms_add_control_edge: null graph");
  const int n = (int)g->g.nodes.size();
  NEED(from >= 0 && from < n && to >= 0 && to < n && from != to, "lms_add_control_edge: unknown node");
  NEED(!g->g.nodes[to].is_var, "lms_add_control_edge: no control edge into a variable");
  g->g.nodes[to].ctrl_in.push_back(from);
  std::vector<int> gam;
  if (!lms::topo_levels(g->g, gam)) {
    g->g.nodes[to].ctrl_in.pop_back();
    set_error("lms_add_control_edge: edge %d -> %d would close a cycle", from, to);
    return LMS_ECYCLE;
  }
  return LMS_OK;
}
lms_status lms_build_backward(lms_graph* g, int32_t loss_node) {
  NEED(g, "lms_build_backward: null graph");
  return lms::build_backward(g->g, loss_node);
}

lms_status lms_build_update(lms_graph* g, float lr, float momentum, int32_t* n_updates) {
  NEED(g, "lms_build_update: null graph");
  int n = 0;
  const lms_status st = lms::build_update(g->g, lr, momentum, &n);
  if (n_updates) *n_updates = n;
  return st;
}

lms_status lms_params_default(lms_params* p) {
  NEED(p, "lms_params_default: null");
  memset(p, 0, sizeof(*p));
  p->n_tensors = -1;
  p->lb = 1;
  p->ub = 10000;
  p->ctrld_strategy = LMS_CHAIN_RULE;
  p->fuse_distance = -1;
  return LMS_OK;
}
lms_status lms_rewrite(lms_graph* g, const lms_params* p, lms_rewrite_stats* stats) {
  NEED(g && p, "lms_rewrite: null argument");
  return lms::rewrite_graph(g->g, *p, stats);
}
lms_status lms_memory_need(const lms_graph* g, uint64_t* peak_live, uint64_t* arena_bytes) {
  NEED(g, "lms_memory_need: null graph");
  lms::PlanResult pr;
  lms::plan_memory(g->g, 0, false, nullptr, pr);
  if ((int)pr.order.size() != (int)g->g.nodes.size()) { set_error("lms_memory_need: graph has a cycle"); return LMS_ECYCLE; }
  if (peak_live) *peak_live = pr.peak_live;
  if (arena_bytes) *arena_bytes = pr.arena_needed;
  return LMS_OK;
}

lms_status lms_node_count(const lms_graph* g, int32_t* n) {
  NEED(g && n, "lms_node_count: null argument");
  *n = (int32_t)g->g.nodes.size();
  return LMS_OK;
}
lms_status lms_node_info_get(const lms_graph* g, int32_t id, lms_node_info* out) {
  NEED(g && out, "lms_node_info_get: null argument");
  NEED(id >= 0 && id < (int)g->g.nodes.size(), "lms_node_info_get: unknown node");
  const lms::Node& n = g->g.nodes[id];
  memset(out, 0, sizeof(*out));
  out->id = n.id; out->op = n.op; out->phase = n.phase; out->placement = n.placement;
  out->is_variable = n.is_var; out->var_kind = n.var_kind; out->dtype = n.dtype; out->ndim = n.ndim;
  for (int i = 0; i < 5; ++i) out->dims[i] = n.dims[i];
  if (n.label >= 0) out->gamma = n.label;
  else {
    // orders of vertices that existed before rewriting are those of the graph without swap vertices
    lms::Graph base;
    for (const lms::Node& m : g->g.nodes) {
      if (m.op == LMS_OP_SWAP_OUT || m.op == LMS_OP_SWAP_IN) break;   // swap vertices come last; recomputed copies stay
      base.nodes.push_back(m);
    }
    for (lms::Node& m : base.nodes)
      for (int& src : m.in) {
        int s = src;
        while (g->g.nodes[s].op == LMS_OP_SWAP_OUT || g->g.nodes[s].op == LMS_OP_SWAP_IN) s = g->g.nodes[s].in[0];
        src = s;
      }
    std::vector<int> gam;
    lms::topo_levels(base, gam);
    out->gamma = gam[id];
  }
  out->n_inputs = (int)n.in.size();
  out->n_control_inputs = (int)n.ctrl_in.size();
  out->flags = n.attr.flags;
  out->bytes = n.bytes();
  out->workspace_bytes = n.is_var ? 0 : lms::workspace_bytes(g->g, n);
  strncpy(out->name, n.name.c_str(), sizeof(out->name) - 1);
  return LMS_OK;
}
lms_status lms_node_find(const lms_graph* g, const char* name, int32_t* id_out) {
  NEED(g && name && id_out, "lms_node_find: null argument");
  for (const lms::Node& n : g->g.nodes)
    if (n.name == name) { *id_out = n.id; return LMS_OK; }
  set_error("lms_node_find: no node named %s", name);
  return LMS_EINVAL;
}
lms_status lms_node_set_external(lms_graph* g, int32_t id, int32_t external) {
  NEED(g, "lms_node_set_external: null graph");
  NEED(id >= 0 && id < (int)g->g.nodes.size(), "lms_node_set_external: unknown node");
  lms::Node& n = g->g.nodes[id];
  NEED(!n.is_var && n.op != LMS_OP_SWAP_OUT && n.op != LMS_OP_SWAP_IN, "lms_node_set_external: variables and swap operations have no arena block");
  n.external = external != 0;
  return LMS_OK;
}
lms_status lms_node_attr_get(const lms_graph* g, int32_t id, lms_attr* out) {
  NEED(g && out, "lms_node_attr_get: null argument");
  NEED(id >= 0 && id < (int)g->g.nodes.size(), "lms_node_attr_get: unknown node");
  *out = g->g.nodes[id].attr;
  return LMS_OK;
}
static void list_edges(const lms::Graph& g, std::vector<lms_edge_info>& out) {
  for (const lms::Node& n : g.nodes) {
    for (int i = 0; i < (int)n.in.size(); ++i) out.push_back(lms_edge_info{n.in[i], n.id, LMS_READ, i, g.nodes[n.in[i]].bytes()});
    for (int u : n.ctrl_in) out.push_back(lms_edge_info{u, n.id, LMS_CONTROL, -1, 0});
  }
  for (auto& u : g.updates) out.push_back(lms_edge_info{u.first, u.second, LMS_UPDATE, -1, g.nodes[u.first].bytes()});
}
lms_status lms_edge_count(const lms_graph* g, int32_t* n) {
  NEED(g && n, "lms_edge_count: null argument");
  std::vector<lms_edge_info> e;
  list_edges(g->g, e);
  *n = (int32_t)e.size();
  return LMS_OK;
}
lms_status lms_edge_info_get(const lms_graph* g, int32_t index, lms_edge_info* out) {
  NEED(g && out, "lms_edge_info_get: null argument");
  std::vector<lms_edge_info> e;
  list_edges(g->g, e);
  NEED(index >= 0 && index < (int)e.size(), "lms_edge_info_get: index out of range");
  *out = e[index];
  return LMS_OK;
}
lms_status lms_topo_order(const lms_graph* g, int32_t* gamma) {
  NEED(g && gamma, "lms_topo_order: null argument");
  std::vector<int> gam;
  if (!lms::topo_levels(g->g, gam)) { set_error("lms_topo_order: graph has a cycle"); return LMS_ECYCLE; }
  for (size_t i = 0; i < gam.size(); ++i) gamma[i] = gam[i];
  return LMS_OK;
}
lms_status lms_schedule(const lms_graph* g, int32_t* order) {
  NEED(g && order, "lms_schedule: null argument");
  std::vector<int> ord;
  if (!lms::schedule(g->g, ord)) { set_error("lms_schedule: graph has a cycle"); return LMS_ECYCLE; }
  for (size_t i = 0; i < ord.size(); ++i) order[i] = ord[i];
  return LMS_OK;
}

lms_status lms_exec_create(const lms_graph* g, void* arena, uint64_t arena_bytes, void* pinned, uint64_t pinned_bytes,
                           void* compute_stream, void* d2h_stream, void* h2d_stream, uint32_t flags, lms_exec** out) {
  NEED(g && out, "lms_exec_create: null argument");
  return lms::exec_create(g->g, arena, arena_bytes, pinned, pinned_bytes, compute_stream, d2h_stream, h2d_stream, flags,
                          reinterpret_cast<lms::Exec**>(out));
}
lms_status lms_exec_destroy(lms_exec* e) { return lms::exec_destroy(reinterpret_cast<lms::Exec*>(e)); }
lms_status lms_pinned_alloc(uint64_t bytes, void** host_out) {
  NEED(host_out && bytes > 0, "lms_pinned_alloc: NULL argument or zero size");
  *host_out = nullptr;
  return lms::pinned_alloc(bytes, host_out);
}
lms_status lms_pinned_free(void* host) { return lms::pinned_free(host); }
lms_status lms_exec_bind(lms_exec* e, int32_t node, void* device_ptr) {
  return lms::exec_bind(reinterpret_cast<lms::Exec*>(e), node, device_ptr);
}
lms_status lms_exec_set_swap_grid(lms_exec* e, int32_t encode_workgroups, int32_t decode_workgroups) {
  NEED(e, "lms_exec_set_swap_grid: null executor");
  return lms::exec_set_swap_grid(reinterpret_cast<lms::Exec*>(e), encode_workgroups, decode_workgroups);
}
lms_status lms_exec_step(lms_exec* e, float* loss_out, lms_step_stats* stats) {
  return lms::exec_step(reinterpret_cast<lms::Exec*>(e), loss_out, stats);
}
lms_status lms_exec_tensor_ptr(lms_exec* e, int32_t node, void** device_ptr) {
  return lms::exec_tensor_ptr(reinterpret_cast<lms::Exec*>(e), node, device_ptr);
}

lms_status lms_conv_workspace_bytes(const lms_conv_desc* d, int32_t which, uint64_t* bytes) {
  NEED(d && bytes, "lms_conv_workspace_bytes: null argument");
  return lms::standalone_ws(d, which, bytes);
}
lms_status lms_conv_fwd(const lms_conv_desc* d, const void* x, const void* w, const float* scale, const float* shift,
                        const void* res, void* y, void* workspace, void* stream) {
  NEED(d && x && w && y, "lms_conv_fwd: null argument");
  return lms::standalone_conv(d, LMS_CONV_FWD, x, w, scale, shift, res, nullptr, y, workspace, stream);
}
lms_status lms_conv_dgrad(const lms_conv_desc* d, const void* dy, const void* w, const float* scale, const void* addend,
                          const void* mask, void* dx, void* workspace, void* stream) {
  NEED(d && dy && w && dx, "lms_conv_dgrad: null argument");
  return lms::standalone_conv(d, LMS_CONV_DGRAD_K, dy, w, scale, nullptr, addend, mask, dx, workspace, stream);
}
lms_status lms_conv_wgrad(const lms_conv_desc* d, const void* x, const void* dy, float* dw, void* workspace, void* stream) {
  NEED(d && x && dy && dw, "lms_conv_wgrad: null argument");
  return lms::standalone_conv(d, LMS_CONV_WGRAD_K, x, dy, nullptr, nullptr, nullptr, nullptr, dw, workspace, stream);
}

lms_status lms_conv_wgrad_bias(const lms_conv_desc* d, const void* x, const void* dy, float* dw, float* dbias, void* workspace,
                               void* stream) {
  NEED(d && x && dy && dw && dbias, "lms_conv_wgrad_bias: null argument");
  return lms::standalone_conv(d, LMS_CONV_WGRAD_BIAS_K, x, dy, nullptr, dbias, nullptr, nullptr, dw, workspace, stream);
}
lms_status lms_swap_encode_staged(void* dst_host, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end, void* stage, int32_t w,
                                  void* stream) {
  NEED(dst_host && src && numel % 8 == 0, "lms_swap_encode_staged: null pointer or element count not a multiple of 8");
  NEED((((uintptr_t)dst_host | (uintptr_t)src | (uintptr_t)stage) & 15) == 0, "lms_swap_encode_staged: pointers must be 16-byte aligned");
  return lms::swap_codec_staged(dst_host, src, numel, slot_begin, slot_end, stage, w, true, stream);
}
lms_status lms_swap_decode_staged(void* dst, const void* src_host, uint64_t numel, int64_t slot_begin, int64_t slot_end, const void* stage,
                                  int32_t w, void* stream) {
  NEED(dst && src_host && numel % 8 == 0, "lms_swap_decode_staged: null pointer or element count not a multiple of 8");
  NEED((((uintptr_t)dst | (uintptr_t)src_host | (uintptr_t)stage) & 15) == 0, "lms_swap_decode_staged: pointers must be 16-byte aligned");
  return lms::swap_codec_staged(dst, src_host, numel, slot_begin, slot_end, const_cast<void*>(stage), w, false, stream);
}
uint64_t lms_swap_staging_bytes(void) { return lms::swap_staging_bytes(); }
lms_status lms_device_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  NEED(dst && src && (bytes % 16) == 0, "lms_device_copy: null pointer or size not a multiple of 16");
  return lms::device_copy(dst, src, bytes, stream);
}

lms_status lms_mfma_probe(uint32_t iters, int32_t random_operands, uint64_t* flops, void* stream) {
  NEED(iters > 0 && iters <= (1u << 22), "lms_mfma_probe: iters must be in 1 .. 2^22");
  return lms::mfma_probe(iters, random_operands != 0, flops, stream);
}

lms_status lms_swap_encoded_bytes(uint64_t numel, uint64_t* bytes) {
  NEED(bytes, "lms_swap_encoded_bytes: null pointer");
  *bytes = lms::swap_encoded_bytes(numel);
  return LMS_OK;
}
lms_status lms_swap_encode(void* dst_host, const void* src, uint64_t numel, void* stream) {
  NEED(dst_host && src && numel % 8 == 0, "lms_swap_encode: null pointer or element count not a multiple of 8");
  NEED(((uintptr_t)dst_host & 15) == 0 && ((uintptr_t)src & 15) == 0, "lms_swap_encode: pointers must be 16-byte aligned");
  return lms::swap_codec(dst_host, src, numel, true, stream);
}
lms_status lms_swap_decode(void* dst, const void* src_host, uint64_t numel, void* stream) {
  NEED(dst && src_host && numel % 8 == 0, "lms_swap_decode: null pointer or element count not a multiple of 8");
  NEED(((uintptr_t)dst & 15) == 0 && ((uintptr_t)src_host & 15) == 0, "lms_swap_decode: pointers must be 16-byte aligned");
  return lms::swap_codec(dst, src_host, numel, false, stream);
}
lms_status lms_swap_moved_bytes(const void* host, uint64_t numel, uint64_t* bytes) {
  NEED(host && bytes, "lms_swap_moved_bytes: null pointer");
  *bytes = lms::swap_encoded_moved_bytes(host, numel);
  return LMS_OK;
}

}  // extern "C"
