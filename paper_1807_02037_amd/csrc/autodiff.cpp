// Backward phase of Section 3.3: for every forward operation f_i with a learnable parameter
// upstream, gradient operations that read f_i's inputs / output (the forward-to-backward edges
// that the rewriting later acts on).
//
// Gradient operations that end in an element-wise tail are emitted lazily so that the tail can be
// fused into them: the data gradient of a convolution is only created when the tensor it flows
// into is finalised, and then it also adds the gradients arriving by other paths (residual
// shortcuts) and applies the ReLU mask of the producer of that tensor.
#include <map>
#include <string>

#include "graph.hpp"

namespace lms {

namespace {

struct Pending {
  int op;
  std::vector<int> ins;
  lms_attr attr;
  bool takes_addend;
  std::string name;
};
struct Contrib {
  bool pending;
  int tensor;
  Pending p;
};

struct Builder {
  Graph& g;
  std::vector<char> learn;
  std::map<int, std::vector<Contrib>> contrib;
  lms_status st = LMS_OK;

  explicit Builder(Graph& gr) : g(gr) {}

  int emit(const std::string& name, int op, const lms_attr* a, const std::vector<int>& ins) {
    int id = -1;
    lms_status s = add_op(g, name.c_str(), op, a, (int)ins.size(), ins.data(), LMS_BWD, &id);
    if (s != LMS_OK && st == LMS_OK) st = s;
    return id;
  }
  void give_tensor(int v, int t) {
    if (learn[v]) contrib[v].push_back(Contrib{false, t, {}});
  }
  void give_pending(int v, Pending p) {
    if (learn[v]) contrib[v].push_back(Contrib{true, -1, std::move(p)});
  }
  int emit_pending(Pending& p, int addend, int mask) {
    lms_attr a = p.attr;
    std::vector<int> ins = p.ins;
    if (addend >= 0) { a.flags |= LMS_F_ADDEND; ins.push_back(addend); }
    if (mask >= 0) {
      a.flags |= LMS_F_MASK;
      if (p.op != LMS_OP_MAXPOOL_BWD) ins.push_back(mask);   // max-pool masks with its own x input
    }
    return emit(p.name, p.op, &a, ins);
  }

  // Gradient with respect to the pre-activation of forward node v: sum of everything that was
  // contributed to v's output, masked by v's output if v ends in a ReLU.
  int finalize(int v) {
    const Node& nv = g.nodes[v];
    const bool need_mask = nv.op == LMS_OP_CONV && (nv.attr.flags & LMS_F_RELU);
    const int mask = need_mask ? v : -1;
    std::vector<Contrib>& cs = contrib[v];
    std::vector<int> tens;
    std::vector<Pending*> pend;
    for (Contrib& c : cs) {
      if (c.pending) pend.push_back(&c.p);
      else tens.push_back(c.tensor);
    }
    const std::string gname = nv.name + "/grad";
    if (pend.empty()) {
      if (tens.size() == 1 && !need_mask) return tens[0];
      lms_attr a{};
      a.filt[0] = a.filt[1] = a.filt[2] = 1;
      a.stride = 1;
      std::vector<int> ins(tens.begin(), tens.begin() + std::min<size_t>(4, tens.size()));
      for (size_t i = 4; i < tens.size(); ++i) {   // more than four: chain plain sums first
        int s = emit(gname + "/part" + std::to_string(i), LMS_OP_GRAD_SUM, &a, {ins[0], tens[i]});
        ins[0] = s;
      }
      if (need_mask) { a.flags |= LMS_F_MASK; ins.push_back(mask); }
      return emit(gname, LMS_OP_GRAD_SUM, &a, ins);
    }
    int acc = -1;
    lms_attr plain{};
    plain.filt[0] = plain.filt[1] = plain.filt[2] = 1;
    plain.stride = 1;
    for (size_t i = 0; i < tens.size(); ++i)
      acc = (acc < 0) ? tens[i] : emit(gname + "/sum" + std::to_string(i), LMS_OP_GRAD_SUM, &plain, {acc, tens[i]});
    for (size_t i = 0; i < pend.size(); ++i) {
      Pending& p = *pend[i];
      const bool last = i + 1 == pend.size();
      if (!last) p.name += "/part";
      if (p.takes_addend || acc < 0) {
        acc = emit_pending(p, p.takes_addend ? acc : -1, last ? mask : -1);
      } else {
        int t = emit_pending(p, -1, -1);
        lms_attr a = plain;
        std::vector<int> ins{acc, t};
        if (last && need_mask) { a.flags |= LMS_F_MASK; ins.push_back(mask); }
        acc = emit(gname + (last ? "" : "/sum_p" + std::to_string(i)), LMS_OP_GRAD_SUM, &a, ins);
      }
    }
    return acc;
  }
};

bool learnable(const Node& n) { return n.is_var && n.var_kind == LMS_VAR_PARAM; }

}  // namespace

lms_status build_backward(Graph& g, int loss_node) {
  if (loss_node < 0 || loss_node >= (int)g.nodes.size()) { set_error("lms_build_backward: bad loss node"); return LMS_EINVAL; }
  const Node& ln = g.nodes[loss_node];
  if (ln.op != LMS_OP_MSE && ln.op != LMS_OP_SOFTMAX_CE) { set_error("lms_build_backward: node %d is not a loss", loss_node); return LMS_EINVAL; }
  Builder b(g);
  const int n_fwd = (int)g.nodes.size();
  b.learn.assign(n_fwd, 0);
  for (int v = 0; v < n_fwd; ++v) {
    const Node& n = g.nodes[v];
    if (learnable(n)) b.learn[v] = 1;
    else if (!n.is_var && n.phase == LMS_FWD)
      for (int u : n.in)
        if (b.learn[u]) b.learn[v] = 1;
  }
  b.learn.resize(n_fwd, 0);
  auto grad_name = [&](int var) { return "grad/" + g.nodes[var].name; };

  for (int v = loss_node; v >= 0; --v) {
    // copy what is needed: emitting nodes reallocates g.nodes
    const Node n = g.nodes[v];
    if (n.is_var || n.phase != LMS_FWD || !b.learn[v]) continue;
    if (v != loss_node && b.contrib.find(v) == b.contrib.end()) continue;
    const uint32_t f = n.attr.flags;
    lms_attr base{};
    base.filt[0] = base.filt[1] = base.filt[2] = 1;
    base.stride = 1;
    if (n.op == LMS_OP_MSE || n.op == LMS_OP_SOFTMAX_CE) {
      Pending p{n.op == LMS_OP_MSE ? LMS_OP_MSE_GRAD : LMS_OP_SOFTMAX_CE_GRAD, {n.in[0], n.in[1]}, base, false, "loss/grad"};
      b.give_pending(n.in[0], p);
      continue;
    }
    const int dz = b.finalize(v);
    if (b.st != LMS_OK) return b.st;
    switch (n.op) {
      case LMS_OP_CONV: {
        const int x = n.in[0], w = n.in[1];
        lms_attr a = base;
        for (int i = 0; i < 3; ++i) a.filt[i] = n.attr.filt[i];
        a.stride = n.attr.stride;
        a.pad = n.attr.pad;
        int slot = 2, scale = -1;
        if (f & LMS_F_AFFINE) {
          scale = n.in[slot];
          const int shift = n.in[slot + 1];
          slot += 2;
          const int raw = b.emit(n.name + "/dw_raw", LMS_OP_CONV_WGRAD, &a, {x, dz});
          if (learnable(g.nodes[w])) b.emit(grad_name(w), LMS_OP_SCALE_COLS, &base, {raw, scale});
          if (learnable(g.nodes[scale])) b.emit(grad_name(scale), LMS_OP_DOT_COLS, &base, {raw, w});
          if (learnable(g.nodes[shift])) b.emit(grad_name(shift), LMS_OP_COLSUM, &base, {dz});
        } else {
          if (learnable(g.nodes[w])) b.emit(grad_name(w), LMS_OP_CONV_WGRAD, &a, {x, dz});
          if (f & LMS_F_BIAS) {
            const int bias = n.in[slot++];
            if (learnable(g.nodes[bias])) b.emit(grad_name(bias), LMS_OP_COLSUM, &base, {dz});
          }
        }
        if (f & LMS_F_RES) b.give_tensor(n.in[slot], dz);
        if (b.learn[x]) {
          Pending p{LMS_OP_CONV_DGRAD, {dz, w}, a, true, n.name + "/dgrad"};
          if (scale >= 0) { p.attr.flags |= LMS_F_AFFINE; p.ins.push_back(scale); }
          const Node& nx = g.nodes[x];
          p.attr.ndim_out = nx.ndim;
          for (int i = 0; i < nx.ndim; ++i) p.attr.out_dims[i] = nx.dims[i];
          b.give_pending(x, p);
        }
        break;
      }
      case LMS_OP_TCONV: {
        const int x = n.in[0], w = n.in[1];
        if (learnable(g.nodes[w])) b.emit(grad_name(w), LMS_OP_TCONV_WGRAD, &base, {x, dz});
        if (b.learn[x]) {
          Pending p{LMS_OP_TCONV_DGRAD, {dz, w}, base, true, n.name + "/dgrad"};
          const Node& nx = g.nodes[x];
          p.attr.ndim_out = nx.ndim;
          for (int i = 0; i < nx.ndim; ++i) p.attr.out_dims[i] = nx.dims[i];
          b.give_pending(x, p);
        }
        break;
      }
      case LMS_OP_MAXPOOL: {
        lms_attr a = n.attr;
        a.flags = 0;
        b.give_pending(n.in[0], Pending{LMS_OP_MAXPOOL_BWD, {dz, n.in[0]}, a, false, n.name + "/bwd"});
        break;
      }
      case LMS_OP_GAP: {
        lms_attr a = base;
        const Node& nx = g.nodes[n.in[0]];
        a.ndim_out = nx.ndim;
        for (int i = 0; i < nx.ndim; ++i) a.out_dims[i] = nx.dims[i];
        b.give_pending(n.in[0], Pending{LMS_OP_GAP_BWD, {dz}, a, false, n.name + "/bwd"});
        break;
      }
      case LMS_OP_CONCAT: {
        int begin = 0;
        for (int j = 0; j < 2; ++j) {
          lms_attr a = base;
          a.c_begin = begin;
          a.c_count = (int)g.nodes[n.in[j]].channels();
          begin += a.c_count;
          b.give_pending(n.in[j], Pending{LMS_OP_SLICE_C, {dz}, a, false, n.name + (j ? "/bwd_b" : "/bwd_a")});
        }
        break;
      }
      default:
        set_error("lms_build_backward: no gradient rule for op %d (%s)", n.op, n.name.c_str());
        return LMS_EINVAL;
    }
    if (b.st != LMS_OK) return b.st;
  }
  return b.st;
}

// Update phase: update/p = p - lr * grad/p for every learnable parameter that has a gradient operation.
lms_status build_update(Graph& g, float lr, float momentum, int* n_updates) {
  int added = 0;
  const int n0 = (int)g.nodes.size();
  for (int v = 0; v < n0; ++v) {
    const Node& p = g.nodes[v];
    if (!p.is_var || p.var_kind != LMS_VAR_PARAM) continue;
    int grad = -1;
    const std::string want = "grad/" + p.name;
    for (int u = 0; u < n0; ++u)
      if (!g.nodes[u].is_var && g.nodes[u].name == want) grad = u;
    if (grad < 0) continue;
    for (const auto& e : g.updates)
      if (e.second == v) { set_error("lms_build_update: %s already has an update edge", p.name.c_str()); return LMS_EINVAL; }
    lms_attr a{};
    a.filt[0] = a.filt[1] = a.filt[2] = 1;
    a.stride = 1;
    a.lr = lr;
    int step = grad;
    const std::string pname = p.name;       // add_variable / add_op may move the node array
    if (momentum > 0.f) {
      int vel = -1;
      int64_t dims[5];
      const int ndim = g.nodes[v].ndim;
      for (int i = 0; i < 5; ++i) dims[i] = g.nodes[v].dims[i];
      lms_status st = add_variable(g, ("velocity/" + pname).c_str(), LMS_F32, ndim, dims, LMS_VAR_CONST, &vel);
      if (st != LMS_OK) return st;
      lms_attr m = a;
      m.lr = momentum;
      const int vin[2] = {vel, grad};
      st = add_op(g, ("update/velocity/" + pname).c_str(), LMS_OP_MOMENTUM, &m, 2, vin, LMS_UPD, &step);
      if (st != LMS_OK) return st;
      g.updates.emplace_back(step, vel);
    }
    const int in[2] = {v, step};
    int id = -1;
    const lms_status st = add_op(g, ("update/" + pname).c_str(), LMS_OP_SGD, &a, 2, in, LMS_UPD, &id);
    if (st != LMS_OK) return st;
    g.updates.emplace_back(id, v);
    ++added;
  }
  if (n_updates) *n_updates = added;
  return LMS_OK;
}

}  // namespace lms
