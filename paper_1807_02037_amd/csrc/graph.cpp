// Graph construction, shape inference and the topological ordering of Definition 2.
#include "graph.hpp"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <queue>

namespace lms {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
const char* get_error() { return g_err; }

// Definition 2 with minimal levels: variables have order 0 and incoming (update) edges do not
// change it; every other vertex is one more than the largest order among the sources of its
// read and control edges.  Kahn's algorithm doubles as the cycle check.
bool topo_levels(const Graph& g, std::vector<int>& gamma) {
  const int n = (int)g.nodes.size();
  gamma.assign(n, 0);
  std::vector<int> indeg(n, 0);
  std::vector<std::vector<int>> succ(n);
  for (const Node& v : g.nodes) {
    if (v.is_var) continue;
    for (int u : v.in) { succ[u].push_back(v.id); ++indeg[v.id]; }
    for (int u : v.ctrl_in) { succ[u].push_back(v.id); ++indeg[v.id]; }
  }
  std::vector<int> ready;
  for (int i = 0; i < n; ++i)
    if (indeg[i] == 0) ready.push_back(i);
  int done = 0;
  while (!ready.empty()) {
    int v = ready.back();
    ready.pop_back();
    ++done;
    const Node& nv = g.nodes[v];
    if (!nv.is_var) {
      int m = 0;
      for (int u : nv.in) m = std::max(m, gamma[u]);
      for (int u : nv.ctrl_in) m = std::max(m, gamma[u]);
      gamma[v] = m + 1;
    }
    for (int s : succ[v])
      if (--indeg[s] == 0) ready.push_back(s);
  }
  return done == n;
}

void adjacency(const Graph& g, std::vector<std::vector<int>>& readers, std::vector<std::vector<int>>& outs) {
  const int n = (int)g.nodes.size();
  readers.assign(n, {});
  outs.assign(n, {});
  for (const Node& v : g.nodes) {
    for (int u : v.in) { readers[u].push_back(v.id); outs[u].push_back(v.id); }
    for (int u : v.ctrl_in) outs[u].push_back(v.id);
  }
  for (int i = 0; i < n; ++i) {
    for (auto* l : {&readers[i], &outs[i]}) {
      std::sort(l->begin(), l->end());
      l->erase(std::unique(l->begin(), l->end()), l->end());
    }
  }
}

void ancestors_of(const Graph& g, int target, std::vector<char>& anc) {
  anc.assign(g.nodes.size(), 0);
  std::vector<int> stack{target};
  while (!stack.empty()) {
    int v = stack.back();
    stack.pop_back();
    const Node& nv = g.nodes[v];
    for (const std::vector<int>* l : {&nv.in, &nv.ctrl_in})
      for (int u : *l)
        if (!anc[u]) { anc[u] = 1; stack.push_back(u); }
  }
}

lms_status add_variable(Graph& g, const char* name, int dtype, int ndim, const int64_t* dims, int kind, int* out) {
  if (!name || ndim < 0 || ndim > 5 || (ndim > 0 && !dims) || dtype < 0 || dtype > LMS_I32) {
    set_error("lms_add_variable: bad argument");
    return LMS_EINVAL;
  }
  Node n;
  n.id = (int)g.nodes.size();
  n.name = name;
  n.op = LMS_OP_VARIABLE;
  n.is_var = true;
  n.var_kind = kind;
  n.dtype = dtype;
  n.ndim = ndim;
  for (int i = 0; i < ndim; ++i) {
    if (dims[i] <= 0) { set_error("lms_add_variable(%s): non-positive extent", name); return LMS_EINVAL; }
    n.dims[i] = dims[i];
  }
  g.nodes.push_back(n);
  if (out) *out = n.id;
  return LMS_OK;
}

static bool same_shape(const Node& a, const Node& b) {
  if (a.ndim != b.ndim) return false;
  for (int i = 0; i < a.ndim; ++i)
    if (a.dims[i] != b.dims[i]) return false;
  return true;
}

static void copy_shape(Node& dst, const Node& src) {
  dst.ndim = src.ndim;
  for (int i = 0; i < 5; ++i) dst.dims[i] = src.dims[i];
}

#define FAIL(...)            \
  do {                       \
    set_error(__VA_ARGS__);  \
    return LMS_EINVAL;       \
  } while (0)

// Number of inputs an operation expects given its flags, and the roles of the optional ones.
static int expected_inputs(int op, uint32_t f, int n_in) {
  switch (op) {
    case LMS_OP_CONV: return 2 + ((f & LMS_F_AFFINE) ? 2 : 0) + ((f & LMS_F_BIAS) ? 1 : 0) + ((f & LMS_F_RES) ? 1 : 0);
    case LMS_OP_CONV_DGRAD:
      return 2 + ((f & LMS_F_AFFINE) ? 1 : 0) + ((f & LMS_F_ADDEND) ? 1 : 0) + ((f & LMS_F_MASK) ? 1 : 0);
    case LMS_OP_TCONV_DGRAD: return 2 + ((f & LMS_F_ADDEND) ? 1 : 0) + ((f & LMS_F_MASK) ? 1 : 0);
    case LMS_OP_CONV_WGRAD: case LMS_OP_TCONV_WGRAD: case LMS_OP_TCONV: case LMS_OP_CONCAT:
    case LMS_OP_MSE: case LMS_OP_SOFTMAX_CE: case LMS_OP_MAXPOOL_BWD: case LMS_OP_SCALE_COLS: case LMS_OP_DOT_COLS:
    case LMS_OP_SGD: case LMS_OP_MOMENTUM:
      return 2;
    case LMS_OP_MAXPOOL: case LMS_OP_GAP: case LMS_OP_COLSUM: case LMS_OP_SWAP_OUT: case LMS_OP_SWAP_IN: return 1;
    case LMS_OP_GAP_BWD: case LMS_OP_SLICE_C: return 1 + ((f & LMS_F_MASK) ? 1 : 0);
    case LMS_OP_MSE_GRAD: case LMS_OP_SOFTMAX_CE_GRAD: return 2 + ((f & LMS_F_MASK) ? 1 : 0);
    case LMS_OP_GRAD_SUM: return n_in;
    default: return -1;
  }
}

lms_status add_op(Graph& g, const char* name, int op, const lms_attr* attr, int n_in, const int* inputs,
                  int phase, int* out) {
  if (!name || n_in < 0 || (n_in > 0 && !inputs)) FAIL("lms_add_op: bad argument");
  Node n;
  n.id = (int)g.nodes.size();
  n.name = name;
  n.op = op;
  n.phase = phase;
  if (attr) n.attr = *attr;
  else { n.attr.filt[0] = n.attr.filt[1] = n.attr.filt[2] = 1; n.attr.stride = 1; }
  const uint32_t f = n.attr.flags;
  for (int i = 0; i < n_in; ++i) {
    if (inputs[i] < 0 || inputs[i] >= n.id) FAIL("lms_add_op(%s): input %d names no earlier node", name, i);
    n.in.push_back(inputs[i]);
  }
  int want = expected_inputs(op, f, n_in);
  if (want < 0) FAIL("lms_add_op(%s): unknown op %d", name, op);
  if (want != n_in) FAIL("lms_add_op(%s): op %d with flags 0x%x takes %d inputs, got %d", name, op, f, want, n_in);
  auto IN = [&](int i) -> const Node& { return g.nodes[n.in[i]]; };
  // activations are bf16; a graph whose input batch and filters are fp32 runs in the fp32 check mode: every
  // activation then takes the type of the operation's first input
  n.dtype = (n_in > 0 && IN(0).dtype == LMS_F32) ? LMS_F32 : LMS_BF16;
  switch (op) {
    case LMS_OP_CONV: {
      const Node& x = IN(0);
      const Node& w = IN(1);
      int nsp = x.nsp();
      if (nsp < 2 || nsp > 3 || w.ndim != nsp + 2) FAIL("conv(%s): x must be NHWC/NDHWC and w (filter..., C, K)", name);
      if (x.dtype == LMS_I32 || w.dtype != x.dtype) FAIL("conv(%s): x and w must both be bf16 (or both fp32: check mode)", name);
      if (w.dims[nsp] != x.channels()) FAIL("conv(%s): filter C %lld != input C %lld", name, (long long)w.dims[nsp], (long long)x.channels());
      if (n.attr.stride < 1 || n.attr.pad < 0) FAIL("conv(%s): bad stride/pad", name);
      n.ndim = x.ndim;
      n.dims[0] = x.dims[0];
      for (int i = 0; i < nsp; ++i) {
        n.attr.filt[i] = (int)w.dims[i];
        int64_t o = (x.dims[1 + i] + 2 * n.attr.pad - w.dims[i]) / n.attr.stride + 1;
        if (x.dims[1 + i] + 2 * n.attr.pad < w.dims[i] || o <= 0) FAIL("conv(%s): empty output", name);
        n.dims[1 + i] = o;
      }
      if (nsp == 2) n.attr.filt[2] = 1;
      n.dims[nsp + 1] = w.dims[nsp + 1];
      n.attr.cout = (int)w.dims[nsp + 1];
      int slot = 2;
      if (f & LMS_F_AFFINE) {
        if ((f & LMS_F_BIAS)) FAIL("conv(%s): AFFINE and BIAS are exclusive", name);
        for (int j = 0; j < 2; ++j, ++slot)
          if (IN(slot).dtype != LMS_F32 || IN(slot).numel() != n.attr.cout) FAIL("conv(%s): scale/shift must be fp32 [K]", name);
      }
      if (f & LMS_F_BIAS) {
        if (IN(slot).dtype != LMS_F32 || IN(slot).numel() != n.attr.cout) FAIL("conv(%s): bias must be fp32 [K]", name);
        ++slot;
      }
      if (f & LMS_F_RES) {
        if (!same_shape(IN(slot), n) || IN(slot).dtype != n.dtype) FAIL("conv(%s): residual shape or type differs from output", name);
      }
      break;
    }
    case LMS_OP_CONV_DGRAD: case LMS_OP_TCONV_DGRAD: {
      const Node& dy = IN(0);
      const Node& w = IN(1);
      int nsp = dy.nsp();
      if (n.attr.ndim_out != dy.ndim) FAIL("dgrad(%s): attr.out_dims must give the input-gradient shape", name);
      n.ndim = dy.ndim;
      for (int i = 0; i < n.ndim; ++i) n.dims[i] = n.attr.out_dims[i];
      for (int i = 0; i < nsp; ++i) n.attr.filt[i] = (int)w.dims[i];
      if (nsp == 2) n.attr.filt[2] = 1;
      if (w.ndim != nsp + 2 || w.dims[nsp] != n.channels() || w.dims[nsp + 1] != dy.channels())
        FAIL("dgrad(%s): filter does not match dy / dx channels", name);
      for (int i = 0; i < nsp; ++i) {
        int64_t o = (op == LMS_OP_TCONV_DGRAD) ? n.dims[1 + i] * 2
                                                : (n.dims[1 + i] + 2 * n.attr.pad - w.dims[i]) / n.attr.stride + 1;
        if (o != dy.dims[1 + i]) FAIL("dgrad(%s): dy extent %d inconsistent with dx shape", name, i);
      }
      int slot = 2;
      if (op == LMS_OP_CONV_DGRAD && (f & LMS_F_AFFINE)) ++slot;
      if (f & LMS_F_ADDEND) { if (!same_shape(IN(slot), n)) FAIL("dgrad(%s): addend shape", name); ++slot; }
      if (f & LMS_F_MASK) { if (!same_shape(IN(slot), n)) FAIL("dgrad(%s): mask shape", name); }
      break;
    }
    case LMS_OP_CONV_WGRAD: case LMS_OP_TCONV_WGRAD: {
      const Node& x = IN(0);
      const Node& dy = IN(1);
      int nsp = x.nsp();
      if (dy.ndim != x.ndim) FAIL("wgrad(%s): rank mismatch", name);
      n.dtype = LMS_F32;
      n.ndim = nsp + 2;
      if (op == LMS_OP_TCONV_WGRAD) n.attr.filt[0] = n.attr.filt[1] = 2, n.attr.filt[2] = (nsp == 3 ? 2 : 1);
      for (int i = 0; i < nsp; ++i) n.dims[i] = n.attr.filt[i];
      n.dims[nsp] = x.channels();
      n.dims[nsp + 1] = dy.channels();
      for (int i = 0; i < nsp; ++i) {
        int64_t o = (op == LMS_OP_TCONV_WGRAD) ? x.dims[1 + i] * 2
                                                : (x.dims[1 + i] + 2 * n.attr.pad - n.attr.filt[i]) / n.attr.stride + 1;
        if (o != dy.dims[1 + i]) FAIL("wgrad(%s): dy extent %d inconsistent with x and filter", name, i);
      }
      break;
    }
    case LMS_OP_TCONV: {
      const Node& x = IN(0);
      const Node& w = IN(1);
      int nsp = x.nsp();
      if (w.ndim != nsp + 2 || w.dims[nsp] != x.channels()) FAIL("tconv(%s): filter mismatch", name);
      for (int i = 0; i < nsp; ++i)
        if (w.dims[i] != 2) FAIL("tconv(%s): only window 2 stride 2", name);
      n.ndim = x.ndim;
      n.dims[0] = x.dims[0];
      for (int i = 0; i < nsp; ++i) n.dims[1 + i] = 2 * x.dims[1 + i], n.attr.filt[i] = 2;
      if (nsp == 2) n.attr.filt[2] = 1;
      n.dims[nsp + 1] = w.dims[nsp + 1];
      n.attr.cout = (int)w.dims[nsp + 1];
      n.attr.stride = 2;
      n.attr.pad = 0;
      break;
    }
    case LMS_OP_MAXPOOL: {
      const Node& x = IN(0);
      int nsp = x.nsp();
      int win = n.attr.filt[0];
      if (win < 1 || n.attr.stride < 1 || n.attr.pad >= win) FAIL("maxpool(%s): bad window", name);
      n.ndim = x.ndim;
      n.dims[0] = x.dims[0];
      for (int i = 0; i < nsp; ++i) {
        n.attr.filt[i] = win;
        n.dims[1 + i] = (x.dims[1 + i] + 2 * n.attr.pad - win) / n.attr.stride + 1;
        if (n.dims[1 + i] <= 0) FAIL("maxpool(%s): empty output", name);
      }
      if (nsp == 2) n.attr.filt[2] = 1;
      n.dims[nsp + 1] = x.channels();
      break;
    }
    case LMS_OP_MAXPOOL_BWD: copy_shape(n, IN(1)); break;
    case LMS_OP_GAP: {
      const Node& x = IN(0);
      copy_shape(n, x);
      for (int i = 0; i < x.nsp(); ++i) n.dims[1 + i] = 1;
      break;
    }
    case LMS_OP_GAP_BWD: {
      if (n.attr.ndim_out != IN(0).ndim) FAIL("gap_bwd(%s): attr.out_dims must give the input shape", name);
      n.ndim = n.attr.ndim_out;
      for (int i = 0; i < n.ndim; ++i) n.dims[i] = n.attr.out_dims[i];
      break;
    }
    case LMS_OP_CONCAT: {
      const Node& a = IN(0);
      const Node& b = IN(1);
      if (a.ndim != b.ndim) FAIL("concat(%s): rank mismatch", name);
      for (int i = 0; i + 1 < a.ndim; ++i)
        if (a.dims[i] != b.dims[i]) FAIL("concat(%s): shape mismatch", name);
      copy_shape(n, a);
      n.dims[a.ndim - 1] = a.channels() + b.channels();
      break;
    }
    case LMS_OP_SLICE_C: {
      const Node& x = IN(0);
      if (n.attr.c_begin < 0 || n.attr.c_count <= 0 || n.attr.c_begin + n.attr.c_count > x.channels())
        FAIL("slice(%s): channel range", name);
      copy_shape(n, x);
      n.dims[x.ndim - 1] = n.attr.c_count;
      break;
    }
    case LMS_OP_MSE:
      if (!same_shape(IN(0), IN(1))) FAIL("mse(%s): target shape differs", name);
      n.dtype = LMS_F32; n.ndim = 1; n.dims[0] = 1;
      break;
    case LMS_OP_SOFTMAX_CE:
      if (IN(1).dtype != LMS_I32 || IN(1).numel() * IN(0).channels() != IN(0).numel()) FAIL("softmax_ce(%s): labels must be int32, one per row", name);
      n.dtype = LMS_F32; n.ndim = 1; n.dims[0] = 1;
      break;
    case LMS_OP_MSE_GRAD: case LMS_OP_SOFTMAX_CE_GRAD: copy_shape(n, IN(0)); break;
    case LMS_OP_GRAD_SUM: {
      int ng = n_in - ((f & LMS_F_MASK) ? 1 : 0);
      if (ng < 1 || ng > 4) FAIL("grad_sum(%s): 1..4 gradients", name);
      for (int i = 1; i < n_in; ++i)
        if (!same_shape(IN(0), IN(i))) FAIL("grad_sum(%s): shapes differ", name);
      copy_shape(n, IN(0));
      break;
    }
    case LMS_OP_COLSUM:
      n.dtype = LMS_F32; n.ndim = 1; n.dims[0] = IN(0).channels();
      break;
    case LMS_OP_SCALE_COLS:
      copy_shape(n, IN(0)); n.dtype = LMS_F32;
      break;
    case LMS_OP_DOT_COLS:
      n.dtype = LMS_F32; n.ndim = 1; n.dims[0] = IN(0).channels();
      break;
    case LMS_OP_SWAP_OUT: case LMS_OP_SWAP_IN:
      copy_shape(n, IN(0)); n.dtype = IN(0).dtype; n.placement = LMS_HOST;
      break;
    case LMS_OP_SGD:
      if (IN(0).dtype == LMS_I32 || IN(1).dtype != LMS_F32 || IN(0).numel() != IN(1).numel()) FAIL("sgd(%s): needs a parameter and its fp32 gradient of the same size", name);
      copy_shape(n, IN(0)); n.dtype = IN(0).dtype;
      break;
    case LMS_OP_MOMENTUM:
      if (IN(0).dtype != LMS_F32 || IN(1).dtype != LMS_F32 || IN(0).numel() != IN(1).numel()) FAIL("momentum(%s): needs an fp32 velocity and an fp32 gradient of the same size", name);
      copy_shape(n, IN(0)); n.dtype = LMS_F32;
      break;
    default: FAIL("lms_add_op(%s): unknown op %d", name, op);
  }
  g.nodes.push_back(n);
  if (out) *out = n.id;
  return LMS_OK;
}

}  // namespace lms
