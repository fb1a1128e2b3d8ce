// Graph rewriting for large-model support (Section 4; parameters of Table 2, Section 5.1).
//
// rewrite_graph selects the tensors to swap by a breadth-first walk from the input variables,
// inserts one swap-out per tensor (Eq. 2, fused swap-outs of 4.2.2), one swap-in per consumer or
// per group of close consumers (Eq. 5, 4.2.3), and a control edge from a control operation chosen
// by the direct-order strategy (Algorithm 1), the chain-rule strategy (Algorithm 2) or this
// library's budget-driven placement.  Orders of existing vertices are not recomputed; a swap-out
// is labelled gamma(producer)+1 and a swap-in gamma(control op)+1 as in Figure 3.
#include <algorithm>
#include <climits>
#include <cstring>

#include "graph.hpp"

namespace lms {

namespace {

struct Selection {
  int u;
  std::vector<int> cons;
};

struct Context {
  const Graph& g;            // the graph before rewriting: all searches run on it
  std::vector<int> gam;
  std::vector<std::vector<int>> readers, outs;
  std::vector<std::vector<int>> by_level;
  std::vector<int> order, pos;   // execution order of the graph before rewriting
  explicit Context(const Graph& gr) : g(gr) {}
};

// Valid control operations for a swap-in of u's tensor before consumer v (Section 4.3:
// gamma(swap-out) < gamma(g) < gamma(v)), in execution order.
std::vector<int> valid_controls(const Context& c, int u, int v) {
  std::vector<int> cand;
  for (int q = c.pos[u] + 1; q < c.pos[v]; ++q) {
    const int f = c.order[q];
    const Node& nf = c.g.nodes[f];
    if (nf.is_var || c.gam[f] <= c.gam[u] || c.gam[f] >= c.gam[v]) continue;
    cand.push_back(f);
  }
  return cand;
}

// `list` holds one name or several separated by commas: true if s starts with (prefix) or equals (!prefix) one of them.
bool in_name_list(const std::string& s, const char* list, bool prefix) {
  if (!list) return false;
  const char* a = list;
  while (true) {
    const char* e = strchr(a, ',');
    const size_t len = e ? (size_t)(e - a) : strlen(a);
    if (len > 0 && (prefix ? s.compare(0, len, a, len) == 0 : (s.size() == len && s.compare(0, len, a, len) == 0))) return true;
    if (!e) return false;
    a = e + 1;
  }
}

bool type_scope_ok(const Node& n, const lms_params& p) {
  const uint32_t bit = 1u << n.op;
  if (p.incl_types && !(p.incl_types & bit)) return false;
  if (p.incl_scopes && p.incl_scopes[0] && !in_name_list(n.name, p.incl_scopes, true)) return false;
  if (p.excl_types & bit) return false;
  if (in_name_list(n.name, p.excl_scopes, true)) return false;
  return true;
}

// Section 5.1: breadth-first from the input variables through forward operations; a tensor is
// swapped if some consumer is a backward operation (or, with swap_branches, a forward operation
// further than branch_threshold) more than one order away.
std::vector<Selection> select(const Context& c, const lms_params& p, int limit) {
  const Graph& g = c.g;
  std::vector<int> level;
  for (const Node& n : g.nodes) {
    if (p.starting_op_names) { if (in_name_list(n.name, p.starting_op_names, false)) level.push_back(n.id); }
    else if (n.is_var && n.var_kind == LMS_VAR_INPUT) level.push_back(n.id);
  }
  if (level.empty() && !p.starting_op_names)
    for (const Node& n : g.nodes)
      if (n.is_var) level.push_back(n.id);
  std::vector<char> seen(g.nodes.size(), 0);
  for (int v : level) seen[v] = 1;
  std::vector<Selection> picked;
  while (!level.empty()) {
    std::vector<int> next;
    for (int u : level) {
      const Node& nu = g.nodes[u];
      if (!nu.is_var && nu.phase == LMS_FWD && type_scope_ok(nu, p)) {
        Selection s{u, {}};
        for (int v : c.readers[u]) {
          const Node& nv = g.nodes[v];
          const int d = c.gam[v] - c.gam[u];
          if (nv.is_var || d <= 1) continue;
          if (nv.phase == LMS_BWD || (p.swap_branches && nv.phase == LMS_FWD && d > p.branch_threshold)) s.cons.push_back(v);
        }
        if (!s.cons.empty()) {
          picked.push_back(std::move(s));
          if (limit >= 0 && (int)picked.size() >= limit) { picked.resize(limit); return picked; }
        }
      }
      for (int v : c.readers[u]) {
        const Node& nv = g.nodes[v];
        if (!seen[v] && !nv.is_var && nv.phase == LMS_FWD) { seen[v] = 1; next.push_back(v); }
      }
    }
    std::sort(next.begin(), next.end());
    level.swap(next);
  }
  if (limit >= 0 && (int)picked.size() > limit) picked.resize(limit);
  return picked;
}

// Algorithm 1.  Candidates at distance i from f2, i = lo..hi, walking back towards f1.
int direct_order(const Context& c, const std::vector<char>& anc_f2, int f1, int f2, int lo, int hi, bool need_reach) {
  const long low = std::max<long>((long)c.gam[f2] - hi + 1, c.gam[f1]);
  for (long i = lo; i <= hi; ++i) {
    const long k = (long)c.gam[f2] - i;
    if (k <= low) return -1;
    if (k >= (long)c.by_level.size()) continue;
    for (int f : c.by_level[k])            // ascending id: GET takes the lowest
      if (!need_reach || anc_f2[f]) return f;
  }
  return -1;
}

// Chain-rule strategy (Section 4.3, Algorithm 2), written from its description: the forward operations are visited
// breadth-first from f1, one layer of the walk per depth d = 0, 1, ...; from depth lo on, the first backward
// operation fed by a visited forward operation that lies strictly between f1 and f2 in order and from which f2 is
// reachable is the control operation.  The walk ends without a result at depth hi (or when the forward phase is
// exhausted).  Within a depth, operations are taken in ascending id; an operation is only closed once it has been
// expanded, so it can be met again at a greater depth.
int chain_rule(const Context& c, const std::vector<char>& anc_f2, int f1, int f2, int lo, int hi) {
  const Graph& g = c.g;
  if (lo > hi) return -1;
  std::vector<int> layer{f1}, next;
  std::vector<char> expanded(g.nodes.size(), 0), queued(g.nodes.size(), 0);
  for (int depth = 0; depth < hi && !layer.empty(); ++depth) {
    std::sort(layer.begin(), layer.end());
    next.clear();
    for (int s : layer) {
      if (depth >= lo)
        for (int f : c.outs[s])
          if (g.nodes[f].phase == LMS_BWD && c.gam[f1] < c.gam[f] && c.gam[f] < c.gam[f2] && anc_f2[f]) return f;
      for (int f : c.outs[s]) {
        const Node& nf = g.nodes[f];
        if (nf.phase != LMS_FWD || nf.is_var || expanded[f] || queued[f]) continue;
        queued[f] = 1;
        next.push_back(f);
      }
      expanded[s] = 1;
    }
    for (int f : next) queued[f] = 0;
    layer.swap(next);
  }
  return -1;
}

struct SwapIn {
  int target;                 // earliest consumer of the group
  std::vector<int> consumers;
  int ctrl;
};
struct TensorPlan {
  int u;
  std::vector<SwapIn> ins;
};

// Control operation for a late copy (swap-in or recomputation) of u's tensor ahead of consumer f2: the strategy of
// Section 4.3 the parameters name; if it finds none, the direct-order walk from distance 1 without the reachability
// filter; -1 if that finds none either.
int pick_control(const Context& c, const lms_params& p, int u, int f2, std::vector<char>& anc) {
  ancestors_of(c.g, f2, anc);
  int ctl;
  if (p.ctrld_strategy == LMS_CHAIN_RULE) ctl = chain_rule(c, anc, u, f2, p.lb, p.ub);
  else if (p.ctrld_strategy == LMS_DIRECT_ORDER) ctl = direct_order(c, anc, u, f2, p.lb, p.ub, true);
  else {   // own placement starts from the latest valid operation in execution order; swap-ins are hoisted afterwards
    std::vector<int> cand = valid_controls(c, u, f2);
    ctl = cand.empty() ? -1 : cand.back();
  }
  if (ctl < 0) ctl = direct_order(c, anc, u, f2, 1, p.ub, false);
  return ctl;
}

std::vector<TensorPlan> place(const Context& c, const std::vector<Selection>& sel, const lms_params& p, int& unrewritten) {
  std::vector<TensorPlan> plans;
  std::vector<char> anc;
  const long fuse_d = p.fuse_distance < 0 ? LONG_MAX : p.fuse_distance;
  for (const Selection& s : sel) {
    std::vector<int> cons = s.cons;
    std::sort(cons.begin(), cons.end(), [&](int a, int b) { return c.gam[a] != c.gam[b] ? c.gam[a] < c.gam[b] : a < b; });
    std::vector<std::vector<int>> groups;
    for (int v : cons) {
      if (p.fuse_swapins && !groups.empty() && (long)c.gam[v] - c.gam[groups.back()[0]] <= fuse_d) groups.back().push_back(v);
      else groups.push_back({v});
    }
    TensorPlan tp{s.u, {}};
    for (auto& grp : groups) {
      const int f2 = grp[0];
      const int ctl = pick_control(c, p, s.u, f2, anc);
      if (ctl < 0) { unrewritten += (int)grp.size(); continue; }
      tp.ins.push_back(SwapIn{f2, grp, ctl});
    }
    if (!tp.ins.empty()) plans.push_back(std::move(tp));
  }
  return plans;
}

// Applies the plans to a copy of the original graph.
void apply(const Context& c, const std::vector<TensorPlan>& plans, Graph& out, lms_rewrite_stats& st) {
  out = c.g;
  for (const TensorPlan& tp : plans) {
    const Node& nu = c.g.nodes[tp.u];
    int so = -1;
    add_op(out, (nu.name + "/swap_out").c_str(), LMS_OP_SWAP_OUT, nullptr, 1, &tp.u, LMS_SWAP, &so);
    out.nodes[so].label = c.gam[tp.u] + 1;
    ++st.swap_outs;
    ++st.tensors_swapped;
    st.swapped_bytes_out += nu.bytes();
    for (const SwapIn& si : tp.ins) {
      int sid = -1;
      add_op(out, (nu.name + "/swap_in@" + c.g.nodes[si.target].name).c_str(), LMS_OP_SWAP_IN, nullptr, 1, &so, LMS_SWAP, &sid);
      out.nodes[sid].label = c.gam[si.ctrl] + 1;
      out.nodes[sid].ctrl_in.push_back(si.ctrl);
      for (int v : si.consumers)
        for (int& src : out.nodes[v].in)
          if (src == tp.u) src = sid;
      ++st.swap_ins;
      ++st.control_edges;
      st.swapped_bytes_in += nu.bytes();
    }
  }
}

bool fits(const Graph& g, uint64_t budget, PlanResult* keep = nullptr) {
  PlanResult pr;
  plan_memory(g, budget, false, nullptr, pr, false, false);     // whether it fits: the compact placement decides
  bool ok = pr.fits;
  if (keep) *keep = std::move(pr);
  return ok;
}

// This library's control-edge placement (the paper leaves a cost-aware choice open, Sections 4.3
// and 7): every swap-in starts at the latest valid control operation, then, in the order the
// tensors are needed, each one is moved to the earliest valid control operation with which the
// whole step still fits the budget, so that host-to-device copies start as soon as memory allows.
void hoist_swapins(const Context& c, std::vector<TensorPlan>& plans, uint64_t budget) {
  const std::vector<int>& pos = c.pos;
  struct Ref { int t, s; };
  std::vector<Ref> refs;
  for (int t = 0; t < (int)plans.size(); ++t)
    for (int s = 0; s < (int)plans[t].ins.size(); ++s) refs.push_back(Ref{t, s});
  std::sort(refs.begin(), refs.end(), [&](const Ref& a, const Ref& b) {
    return pos[plans[a.t].ins[a.s].target] < pos[plans[b.t].ins[b.s].target];
  });
  Graph trial;
  for (const Ref& r : refs) {
    SwapIn& si = plans[r.t].ins[r.s];
    const int u = plans[r.t].u, v = si.target;
    const std::vector<int> cand = valid_controls(c, u, v);     // earliest first
    if (cand.empty()) continue;
    const int latest = si.ctrl;
    // earliest candidate that still fits; memory need grows as the swap-in moves earlier
    int lo = 0, hi = (int)cand.size() - 1, best = -1;
    while (lo <= hi) {
      const int mid = (lo + hi) / 2;
      si.ctrl = cand[mid];
      lms_rewrite_stats tmp{};
      apply(c, plans, trial, tmp);
      if (fits(trial, budget)) { best = mid; hi = mid - 1; }
      else lo = mid + 1;
    }
    si.ctrl = (best >= 0 && pos[cand[best]] < pos[latest]) ? cand[best] : latest;
  }
}

bool cheap_op(int op) { return op == LMS_OP_MAXPOOL || op == LMS_OP_CONCAT || op == LMS_OP_GAP; }

void build_context(Context& c) {
  const Graph& g = c.g;
  adjacency(g, c.readers, c.outs);
  schedule(g, c.order);
  c.pos.assign(g.nodes.size(), 0);
  for (int i = 0; i < (int)c.order.size(); ++i) c.pos[c.order[i]] = i;
  int maxlev = 0;
  for (int v : c.gam) maxlev = std::max(maxlev, v);
  c.by_level.assign(maxlev + 1, {});
  for (const Node& n : g.nodes)
    if (!n.is_var) c.by_level[c.gam[n.id]].push_back(n.id);
}

// Recomputation pass (before any swap is inserted): every tensor the selection would swap whose producer is a
// cheap operation gets, per group of late consumers, a copy of the producer with the same inputs, triggered by a
// control edge chosen like a swap-in's; the consumers read the copy.  The copy takes the phase of its first
// consumer, so in the swap pass its inputs are tensors with a late consumer like any other.
lms_status recompute_pass(Graph& g, const lms_params& p, lms_rewrite_stats& st) {
  Context c(g);
  if (!topo_levels(g, c.gam)) { set_error("lms_rewrite: graph has a cycle"); return LMS_ECYCLE; }
  build_context(c);
  std::vector<Selection> cheap;
  for (Selection& s : select(c, p, -1))
    if (cheap_op(g.nodes[s.u].op)) cheap.push_back(std::move(s));
  int unre = 0;
  const std::vector<TensorPlan> plans = place(c, cheap, p, unre);
  st.unrewritten += unre;
  Graph out = g;
  for (const TensorPlan& tp : plans) {
    const Node& nu = g.nodes[tp.u];
    for (const SwapIn& si : tp.ins) {
      int id = -1;
      const lms_status rc = add_op(out, (nu.name + "/recompute@" + g.nodes[si.target].name).c_str(), nu.op, &nu.attr, (int)nu.in.size(),
                                   nu.in.data(), g.nodes[si.target].phase, &id);
      if (rc != LMS_OK) return rc;
      out.nodes[id].label = c.gam[si.ctrl] + 1;
      out.nodes[id].clone_of = tp.u;
      out.nodes[id].ctrl_in.push_back(si.ctrl);
      for (int v : si.consumers)
        for (int& src : out.nodes[v].in)
          if (src == tp.u) src = id;
      ++st.recomputed;
      ++st.control_edges;
    }
  }
  g = std::move(out);
  return LMS_OK;
}

// ---- chained recomputation (the paper names recomputation as future work, Section 7, and gives no rule) --------
// Operation kinds whose output can be produced a second time from the same inputs: every forward operation of this
// library except the losses.
bool recomputable_op(int op) {
  return op == LMS_OP_CONV || op == LMS_OP_TCONV || op == LMS_OP_MAXPOOL || op == LMS_OP_CONCAT || op == LMS_OP_GAP;
}

// Depth rule: over the selected tensors in creation order, a tensor is recomputed if the chain of recomputed
// tensors ending in it stays within `depth`; every other tensor counts as stored (chain length 0).
std::vector<int> recompute_by_depth(const Graph& g, const std::vector<Selection>& all, int depth) {
  std::vector<int> ids;
  for (const Selection& s : all) ids.push_back(s.u);
  std::sort(ids.begin(), ids.end());
  std::vector<int> chain(g.nodes.size(), 0), chosen;
  for (int u : ids) {
    const Node& nu = g.nodes[u];
    if (!recomputable_op(nu.op)) continue;
    int d = 0;
    for (int i : nu.in)
      if (!g.nodes[i].is_var) d = std::max(d, chain[i]);
    if (d + 1 <= depth) { chain[u] = d + 1; chosen.push_back(u); }
  }
  return chosen;
}

// Every chosen tensor gets one late copy of its producer that all its late consumers read.  A copy reads the copies
// of those inputs that are recomputed too and the stored tensors themselves otherwise (the swap pass that follows
// treats those as tensors with a late consumer).  The control operation of u's copy is the one the strategy picks
// for (u, earliest late consumer that u serves, directly or through copies reading it); a copy that feeds another
// copy is never triggered by a later control operation (in creation order) than the copy it feeds.  Copies are
// created in the creation order of their originals, so the executor runs a chain front to back.
// `set`: the producers to recompute, given explicitly (forward tensors; one that nothing late reads, directly or
// through a copy, is ignored); NULL: depth rule.
lms_status recompute_chained_pass(Graph& g, const lms_params& p, int depth, const std::vector<int>* set, lms_rewrite_stats& st) {
  Context c(g);
  if (!topo_levels(g, c.gam)) { set_error("lms_rewrite: graph has a cycle"); return LMS_ECYCLE; }
  build_context(c);
  const std::vector<Selection> all = select(c, p, -1);
  const int n = (int)g.nodes.size();
  std::vector<int> sel_of(n, -1);
  for (int i = 0; i < (int)all.size(); ++i) sel_of[all[i].u] = i;
  std::vector<int> chosen;
  if (set) {
    // a tensor named explicitly need not have a late consumer of its own: a forward tensor that only a recomputed
    // producer reads (the shortcut branch of a residual sum) is recomputed for that copy alone
    for (int u : *set)
      if (u >= 0 && u < n && !g.nodes[u].is_var && (sel_of[u] >= 0 || g.nodes[u].phase == LMS_FWD) && recomputable_op(g.nodes[u].op))
        chosen.push_back(u);
    std::sort(chosen.begin(), chosen.end());
    chosen.erase(std::unique(chosen.begin(), chosen.end()), chosen.end());
  } else {
    chosen = recompute_by_depth(g, all, depth);
  }
  std::vector<char> is_chosen(n, 0);
  for (int u : chosen) is_chosen[u] = 1;
  auto earlier = [&](int a, int b) { return c.gam[a] != c.gam[b] ? c.gam[a] < c.gam[b] : a < b; };
  std::vector<int> target(n, -1), ctrl(n, -1);
  std::vector<std::vector<int>> feeds(n);       // chosen tensors whose producer reads this one
  std::vector<char> anc;
  for (auto it = chosen.rbegin(); it != chosen.rend(); ++it) {
    const int u = *it;
    static const std::vector<int> none;
    const std::vector<int>& cons = sel_of[u] >= 0 ? all[sel_of[u]].cons : none;
    int t = cons.empty() ? -1 : *std::min_element(cons.begin(), cons.end(), earlier);
    for (int w : feeds[u])
      if (ctrl[w] >= 0 && (t < 0 || earlier(target[w], t))) t = target[w];
    if (t < 0) continue;                           // nothing late reads it, directly or through a copy
    int ctl = pick_control(c, p, u, t, anc);
    if (ctl < 0) { st.unrewritten += (int)cons.size(); continue; }
    for (int w : feeds[u])
      if (ctrl[w] >= 0 && ctrl[w] < ctl) ctl = ctrl[w];
    target[u] = t;
    ctrl[u] = ctl;
    for (int i : g.nodes[u].in)
      if (is_chosen[i]) feeds[i].push_back(u);
  }
  Graph out = g;
  std::vector<int> copy(n, -1);
  for (int u : chosen) {
    if (ctrl[u] < 0) continue;
    const Node& nu = g.nodes[u];
    std::vector<int> ins = nu.in;
    int label = c.gam[ctrl[u]] + 1;
    for (int& i : ins)
      if (copy[i] >= 0) { i = copy[i]; label = std::max(label, out.nodes[i].label + 1); }
    int id = -1;
    const lms_status rc = add_op(out, (nu.name + "/recompute@" + g.nodes[target[u]].name).c_str(), nu.op, &nu.attr, (int)ins.size(),
                                 ins.data(), g.nodes[target[u]].phase, &id);
    if (rc != LMS_OK) return rc;
    out.nodes[id].label = label;
    out.nodes[id].clone_of = u;
    out.nodes[id].ctrl_in.push_back(ctrl[u]);
    if (sel_of[u] >= 0)
      for (int v : all[sel_of[u]].cons)
        for (int& src : out.nodes[v].in)
          if (src == u) src = id;
    copy[u] = id;
    ++st.recomputed;
    ++st.control_edges;
  }
  g = std::move(out);
  return LMS_OK;
}

// Rough duration of one operation for the planner's choice between recomputing and swapping: the larger of its
// arithmetic at `tflops` and its tensor traffic at `hbm_gbs`.
double op_seconds(const Graph& g, const Node& n, double tflops, double hbm_gbs) {
  if (n.is_var || n.op == LMS_OP_SWAP_OUT || n.op == LMS_OP_SWAP_IN) return 0.0;
  double bytes = (double)n.bytes();
  for (int i : n.in) bytes += (double)g.nodes[i].bytes();
  double flops = 0.0;
  switch (n.op) {
    case LMS_OP_CONV: case LMS_OP_TCONV: {            // output elements x input channels x taps
      const Node& w = g.nodes[n.in[1]];
      flops = 2.0 * (double)n.numel() * (double)w.numel() / (double)w.dims[w.ndim - 1];
      if (n.op == LMS_OP_TCONV) flops = 2.0 * (double)n.numel() * (double)w.dims[w.ndim - 2];
      break;
    }
    case LMS_OP_CONV_DGRAD: case LMS_OP_TCONV_DGRAD: {
      const Node& w = g.nodes[n.in[1]];
      const Node& dy = g.nodes[n.in[0]];
      flops = 2.0 * (double)dy.numel() * (double)w.numel() / (double)w.dims[w.ndim - 1];
      if (n.op == LMS_OP_TCONV_DGRAD) flops = 2.0 * (double)dy.numel() * (double)w.dims[w.ndim - 2];
      break;
    }
    case LMS_OP_CONV_WGRAD: case LMS_OP_TCONV_WGRAD: {
      const Node& dy = g.nodes[n.in[1]];
      flops = 2.0 * (double)dy.numel() * (double)n.numel() / (double)n.dims[n.ndim - 1];
      if (n.op == LMS_OP_TCONV_WGRAD) flops = 2.0 * (double)dy.numel() * (double)n.dims[n.ndim - 2];
      break;
    }
    default: break;
  }
  return std::max(flops / (tflops * 1e12), bytes / (hbm_gbs * 1e9));
}

// Estimated step time of a rewritten graph: the step played through as the executor runs it.  Operations follow
// one another on the compute stream, swap-outs on a second and swap-ins on a third stream, each in schedule order; a
// node starts when its stream is free, its inputs and control operations are done, and every earlier tenant of its
// arena block (output and workspace, from the memory plan for this budget) has been released: a swapped-out tensor's
// block only when its copy is over.  That last wait is what a plan with too many or too late swap-outs pays, and what
// the sum of the operations against the bytes on the link does not show.  Durations: op_seconds, and the bytes a copy
// is expected to put on the link at the link rate.
double estimate_step_seconds(const Graph& g, const lms_params& p) {
  const double tflops = p.device_tflops > 0 ? p.device_tflops : 800.0;
  const double hbm = p.hbm_gbs > 0 ? p.hbm_gbs : 5000.0;
  const double link = p.link_gbs > 0 ? p.link_gbs : 50.0;
  PlanResult pr;
  plan_memory(g, p.budget_bytes, false, nullptr, pr, p.encoded_swaps != 0);
  const int n = (int)g.nodes.size();
  std::vector<std::vector<int>> readers, outs;
  adjacency(g, readers, outs);
  std::vector<double> finish(n, 0.0);
  double stream_free[3] = {0.0, 0.0, 0.0}, end = 0.0;
  for (int v : pr.order) {
    const Node& nv = g.nodes[v];
    if (nv.is_var) continue;
    double dep = 0.0;
    for (int u : nv.in) dep = std::max(dep, finish[u]);
    for (int u : nv.ctrl_in) dep = std::max(dep, finish[u]);
    auto tenants = [&](const std::vector<int>& prev) {
      for (int m : prev) {
        if (m < 0) { dep = std::max(dep, finish[~m]); continue; }     // a workspace: its operation alone
        dep = std::max(dep, finish[m]);
        for (int r : readers[m]) dep = std::max(dep, finish[r]);
      }
    };
    tenants(pr.prev_tenants[v]);
    tenants(pr.ws_prev_tenants[v]);
    const int stream = nv.op == LMS_OP_SWAP_OUT ? 1 : (nv.op == LMS_OP_SWAP_IN ? 2 : 0);
    double dur;
    if (stream) {
      int src = v;                                   // the tensor behind the swap: the swap-out's input
      while (g.nodes[src].op == LMS_OP_SWAP_OUT || g.nodes[src].op == LMS_OP_SWAP_IN) src = g.nodes[src].in[0];
      dur = expected_link_bytes(g, g.nodes[src], p.encoded_swaps != 0) / (link * 1e9);
    } else {
      dur = op_seconds(g, nv, tflops, hbm);
    }
    finish[v] = std::max(stream_free[stream], dep) + dur;
    stream_free[stream] = finish[v];
    end = std::max(end, finish[v]);
  }
  return end;
}

// The swap pass on g (the graph as it is after any recomputation pass): selection, swap-out / swap-in insertion and
// control-edge placement.  st0: what earlier passes contributed.  With a budget: the smallest number of tensors, in
// breadth-first order, whose rewrite fits; then (own strategy) tensors whose absence the budget does not notice are
// dropped and, if `hoist`, the swap-ins are moved as early as the budget allows.
struct SwapPassResult {
  Graph graph;
  lms_rewrite_stats st{};
  bool ok = true;
};

lms_status swap_pass(const Graph& g, const lms_params& p, const lms_rewrite_stats& st0, bool hoist, SwapPassResult& out) {
  Context c(g);
  if (!topo_levels(g, c.gam)) { set_error("lms_rewrite: graph has a cycle"); return LMS_ECYCLE; }
  build_context(c);
  lms_rewrite_stats st = st0;
  Graph& result = out.graph;
  std::vector<TensorPlan> plans;
  out.ok = true;
  if (p.budget_bytes == 0) {
    int unre = 0;
    plans = place(c, select(c, p, p.n_tensors), p, unre);
    st.unrewritten = st0.unrewritten + unre;
    apply(c, plans, result, st);
  } else {
    const std::vector<Selection> all = select(c, p, -1);
    bool ok = false;
    lms_rewrite_stats best{};
    std::vector<Selection> sel;
    for (int n = 0; n <= (int)all.size() && !ok; ++n) {
      sel.assign(all.begin(), all.begin() + n);
      int unre = 0;
      plans = place(c, sel, p, unre);
      lms_rewrite_stats t = st0;
      t.unrewritten = st0.unrewritten + unre;
      apply(c, plans, result, t);
      ok = fits(result, p.budget_bytes);
      best = t;
    }
    if (ok && p.ctrld_strategy == LMS_OWN && sel.size() > 1) {
      // This library's selection: the prefix that fits usually holds tensors whose absence the budget would not
      // notice (they are not live at the peak).  Drop them, largest first, as long as the step still fits: fewer
      // bytes cross the link for the same budget.
      std::vector<int> by_size(sel.size());
      for (int i = 0; i < (int)sel.size(); ++i) by_size[i] = i;
      std::stable_sort(by_size.begin(), by_size.end(), [&](int a, int b) { return g.nodes[sel[a].u].bytes() > g.nodes[sel[b].u].bytes(); });
      std::vector<char> dropped(sel.size(), 0);
      for (int i : by_size) {
        std::vector<Selection> trial_sel;
        for (int j = 0; j < (int)sel.size(); ++j)
          if (!dropped[j] && j != i) trial_sel.push_back(sel[j]);
        int unre = 0;
        std::vector<TensorPlan> trial_plans = place(c, trial_sel, p, unre);
        lms_rewrite_stats t = st0;
        t.unrewritten = st0.unrewritten + unre;
        Graph trial;
        apply(c, trial_plans, trial, t);
        if (fits(trial, p.budget_bytes)) {
          dropped[i] = 1;
          plans = std::move(trial_plans);
          result = std::move(trial);
          best = t;
        }
      }
    }
    st = best;
    out.ok = ok;
    if (ok && hoist && p.ctrld_strategy == LMS_OWN && !plans.empty()) {
      hoist_swapins(c, plans, p.budget_bytes);
      lms_rewrite_stats t = st0;
      t.unrewritten = st.unrewritten;
      apply(c, plans, result, t);
      st = t;
    }
  }
  PlanResult after;
  fits(result, out.ok ? p.budget_bytes : 0, &after);
  st.peak_live_after = after.peak_live;
  st.arena_needed_after = after.arena_needed;
  out.st = st;
  return LMS_OK;
}

}  // namespace

lms_status rewrite_graph(Graph& g_in, const lms_params& p, lms_rewrite_stats* stats) {
  if (p.lb < 0 || p.ub < 0 || p.ctrld_strategy < 0 || p.ctrld_strategy > LMS_OWN || p.recompute < 0 || p.recompute > 2) {
    set_error("lms_rewrite: bad parameter");
    return LMS_EINVAL;
  }
  for (const Node& n : g_in.nodes)
    if (n.op == LMS_OP_SWAP_OUT || n.op == LMS_OP_SWAP_IN || n.clone_of >= 0) { set_error("lms_rewrite: graph is already rewritten"); return LMS_EINVAL; }
  lms_rewrite_stats base{};
  PlanResult before;
  fits(g_in, 0, &before);
  base.peak_live_before = before.peak_live;
  base.arena_needed_before = before.arena_needed;

  // the caller's graph stays as it is unless the rewrite succeeds
  SwapPassResult chosen;
  if (p.recompute == 2 && p.recompute_depth <= 0 && p.budget_bytes > 0) {
    // Hybrid plan: per tensor recompute, swap or keep: a local search over the set of recomputed tensors, every
    // candidate planned in full (copies, swap pass with hoisted swap-ins, memory plan) and judged by the played-through
    // step (estimate_step_seconds).  The plan with swaps alone comes first (so a budget that swaps can meet is never
    // lost); then every tensor the current plan swaps, largest first, is tried as a recomputed tensor instead (inputs
    // of a copy may have to be swapped or kept longer) and the change stays if the plan still fits and its estimated
    // step is shorter, or as long with fewer bytes over the link; where the change only moved the swap to an input
    // of the copy, that input is tried as well; then every recomputed tensor is tried stored again.  Sweeps repeat,
    // with the tensors turned down before tried anew, until one changes nothing.
    {
      const lms_status rc = swap_pass(g_in, p, base, true, chosen);
      if (rc != LMS_OK) return rc;
    }
    if (!chosen.ok) {
      if (stats) *stats = chosen.st;
      set_error("lms_rewrite: budget %llu bytes is below the %llu bytes the step needs with every tensor swapped",
                (unsigned long long)p.budget_bytes, (unsigned long long)chosen.st.arena_needed_after);
      return LMS_EBUDGET;
    }
    const int n0 = (int)g_in.nodes.size();
    std::vector<int> rec;
    double cur_est = estimate_step_seconds(chosen.graph, p);
    // plans the step with the tensors of `trial` recomputed; 1 = planned and fits, 0 = not usable, < 0 = error
    auto plan_with = [&](const std::vector<int>& trial, SwapPassResult& r, double& est) -> int {
      Graph g = g_in;
      lms_rewrite_stats st = base;
      if (!trial.empty()) {
        const lms_status rc = recompute_chained_pass(g, p, 0, &trial, st);
        if (rc != LMS_OK) return (int)rc;
        if (st.recomputed != (int)trial.size()) return 0;      // no control operation for a copy
      }
      const lms_status rc = swap_pass(g, p, st, true, r);
      if (rc != LMS_OK) return (int)rc;
      if (!r.ok) return 0;
      est = estimate_step_seconds(r.graph, p);
      return 1;
    };
    auto better = [&](double est, const SwapPassResult& r) {
      return est < cur_est || (est == cur_est && r.st.swapped_bytes_out < chosen.st.swapped_bytes_out);
    };
    std::vector<char> tried(n0, 0);
    for (int sweep = 0; sweep < 8; ++sweep) {
      bool changed = false;
      std::vector<int> cand;
      for (const Node& n : chosen.graph.nodes)
        if (n.op == LMS_OP_SWAP_OUT && n.in[0] < n0 && !tried[n.in[0]] && recomputable_op(g_in.nodes[n.in[0]].op)) cand.push_back(n.in[0]);
      std::stable_sort(cand.begin(), cand.end(), [&](int a, int b) { return g_in.nodes[a].bytes() > g_in.nodes[b].bytes(); });
      for (int u : cand) {
        tried[u] = 1;
        std::vector<int> trial = rec;
        trial.push_back(u);
        SwapPassResult r;
        double est = 0.0;
        const int ok = plan_with(trial, r, est);
        if (ok < 0) return (lms_status)ok;
        if (ok && better(est, r)) {
          rec.swap(trial);
          chosen = std::move(r);
          cur_est = est;
          changed = true;
        } else if (ok) {
          // the change only moved the swap to another tensor (an input of the copy, say): look one step further
          // and recompute that one as well
          std::vector<char> swapped_now(n0, 0);
          for (const Node& n : chosen.graph.nodes)
            if (n.op == LMS_OP_SWAP_OUT && n.in[0] < n0) swapped_now[n.in[0]] = 1;
          std::vector<int> moved;
          for (const Node& n : r.graph.nodes)
            if (n.op == LMS_OP_SWAP_OUT && n.in[0] < n0 && !swapped_now[n.in[0]] && recomputable_op(g_in.nodes[n.in[0]].op)) moved.push_back(n.in[0]);
          for (int w : moved) {
            std::vector<int> trial2 = trial;
            trial2.push_back(w);
            SwapPassResult r2;
            double est2 = 0.0;
            const int ok2 = plan_with(trial2, r2, est2);
            if (ok2 < 0) return (lms_status)ok2;
            if (ok2 && better(est2, r2)) {
              rec.swap(trial2);
              chosen = std::move(r2);
              cur_est = est2;
              changed = true;
              break;
            }
          }
        }
      }
      // the other direction: a tensor recomputed so far is stored again (kept or swapped, as the swap pass finds)
      for (size_t i = 0; i < rec.size();) {
        std::vector<int> trial = rec;
        trial.erase(trial.begin() + (long)i);
        SwapPassResult r;
        double est = 0.0;
        const int ok = plan_with(trial, r, est);
        if (ok < 0) return (lms_status)ok;
        if (ok && est < cur_est) {
          tried[rec[i]] = 1;
          rec.swap(trial);
          chosen = std::move(r);
          cur_est = est;
          changed = true;
        } else {
          ++i;
        }
      }
      if (!changed) break;
      // a tensor turned down before may pay now that the plan around it has changed
      std::fill(tried.begin(), tried.end(), 0);
    }
  } else {
    Graph g = g_in;
    lms_rewrite_stats st = base;
    lms_status rc = LMS_OK;
    if (p.recompute == 1) rc = recompute_pass(g, p, st);
    else if (p.recompute == 2) rc = recompute_chained_pass(g, p, p.recompute_depth > 0 ? p.recompute_depth : 2, nullptr, st);
    if (rc != LMS_OK) return rc;
    rc = swap_pass(g, p, st, true, chosen);
    if (rc != LMS_OK) return rc;
    if (!chosen.ok) {
      if (stats) *stats = chosen.st;
      set_error("lms_rewrite: budget %llu bytes is below the %llu bytes the step needs with every tensor swapped",
                (unsigned long long)p.budget_bytes, (unsigned long long)chosen.st.arena_needed_after);
      return LMS_EBUDGET;
    }
  }
  if (p.budget_bytes > 0) chosen.st.estimated_ms = (float)(1e3 * estimate_step_seconds(chosen.graph, p));
  g_in = std::move(chosen.graph);
  if (stats) *stats = chosen.st;
  return LMS_OK;
}

}  // namespace lms
