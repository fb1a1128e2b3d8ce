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

bool starts_with(const std::string& s, const char* prefix) { return prefix && s.compare(0, strlen(prefix), prefix) == 0; }

bool type_scope_ok(const Node& n, const lms_params& p) {
  if (p.incl_type >= 0 && n.op != p.incl_type) return false;
  if (p.incl_scope && !starts_with(n.name, p.incl_scope)) return false;
  if (p.excl_type >= 0 && n.op == p.excl_type) return false;
  if (p.excl_scope && starts_with(n.name, p.excl_scope)) return false;
  return true;
}

// Section 5.1: breadth-first from the input variables through forward operations; a tensor is
// swapped if some consumer is a backward operation (or, with swap_branches, a forward operation
// further than branch_threshold) more than one order away.
std::vector<Selection> select(const Context& c, const lms_params& p, int limit) {
  const Graph& g = c.g;
  std::vector<int> level;
  for (const Node& n : g.nodes) {
    if (p.starting_op_name) { if (n.name == p.starting_op_name) level.push_back(n.id); }
    else if (n.is_var && n.var_kind == LMS_VAR_INPUT) level.push_back(n.id);
  }
  if (level.empty() && !p.starting_op_name)
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

// Algorithm 2.  Level-by-level walk down the forward phase from f1.
int chain_rule(const Context& c, const std::vector<char>& anc_f2, int f1, int f2, int lo, int hi) {
  const Graph& g = c.g;
  std::vector<int> s1{f1}, s2;
  std::vector<char> closed(g.nodes.size(), 0), in_s2(g.nodes.size(), 0);
  while (!s1.empty()) {
    if (hi == 0 || lo > hi) return -1;
    auto it = std::min_element(s1.begin(), s1.end());
    const int s = *it;
    s1.erase(it);
    if (lo <= 0) {
      for (int f : c.outs[s]) {
        const Node& nf = g.nodes[f];
        if (nf.phase == LMS_BWD && c.gam[f] > c.gam[f1] && c.gam[f] < c.gam[f2] && anc_f2[f]) return f;
      }
    }
    for (int f : c.outs[s]) {
      const Node& nf = g.nodes[f];
      if (nf.phase != LMS_FWD || nf.is_var || closed[f] || in_s2[f]) continue;
      in_s2[f] = 1;
      s2.push_back(f);
    }
    closed[s] = 1;
    if (s1.empty()) {
      --lo;
      --hi;
      s1.swap(s2);
      s2.clear();
      for (int f : s1) in_s2[f] = 0;
    }
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
      ancestors_of(c.g, f2, anc);
      int ctl;
      if (p.ctrld_strategy == LMS_CHAIN_RULE) ctl = chain_rule(c, anc, s.u, f2, p.lb, p.ub);
      else if (p.ctrld_strategy == LMS_DIRECT_ORDER) ctl = direct_order(c, anc, s.u, f2, p.lb, p.ub, true);
      else {   // own placement starts from the latest valid operation in execution order; hoisted afterwards
        std::vector<int> cand = valid_controls(c, s.u, f2);
        ctl = cand.empty() ? -1 : cand.back();
      }
      if (ctl < 0) ctl = direct_order(c, anc, s.u, f2, 1, p.ub, false);
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
  plan_memory(g, budget, false, nullptr, pr);
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

}  // namespace

lms_status rewrite_graph(Graph& g_in, const lms_params& p, lms_rewrite_stats* stats) {
  if (p.lb < 0 || p.ub < 0 || p.ctrld_strategy < 0 || p.ctrld_strategy > LMS_OWN) {
    set_error("lms_rewrite: bad parameter");
    return LMS_EINVAL;
  }
  for (const Node& n : g_in.nodes)
    if (n.op == LMS_OP_SWAP_OUT || n.op == LMS_OP_SWAP_IN || n.clone_of >= 0) { set_error("lms_rewrite: graph is already rewritten"); return LMS_EINVAL; }
  lms_rewrite_stats st{};
  PlanResult before;
  fits(g_in, 0, &before);
  st.peak_live_before = before.peak_live;
  st.arena_needed_before = before.arena_needed;
  Graph g = g_in;              // the caller's graph stays as it is unless the rewrite succeeds
  if (p.recompute) {
    const lms_status rc = recompute_pass(g, p, st);
    if (rc != LMS_OK) return rc;
  }
  const lms_rewrite_stats st0 = st;     // what the recomputation pass contributed
  Context c(g);
  if (!topo_levels(g, c.gam)) { set_error("lms_rewrite: graph has a cycle"); return LMS_ECYCLE; }
  build_context(c);

  Graph result;
  std::vector<TensorPlan> plans;
  if (p.budget_bytes == 0) {
    int unre = 0;
    plans = place(c, select(c, p, p.n_tensors), p, unre);
    st.unrewritten = st0.unrewritten + unre;
    apply(c, plans, result, st);
  } else {
    // smallest number of tensors, in breadth-first order, whose rewrite fits the budget
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
    if (!ok) {
      PlanResult after;
      fits(result, 0, &after);
      st.peak_live_after = after.peak_live;
      st.arena_needed_after = after.arena_needed;
      if (stats) *stats = st;
      set_error("lms_rewrite: budget %llu bytes is below the %llu bytes the step needs with every tensor swapped",
                (unsigned long long)p.budget_bytes, (unsigned long long)after.arena_needed);
      return LMS_EBUDGET;
    }
    if (p.ctrld_strategy == LMS_OWN && !plans.empty()) {
      hoist_swapins(c, plans, p.budget_bytes);
      lms_rewrite_stats t = st0;
      t.unrewritten = st.unrewritten;
      apply(c, plans, result, t);
      st = t;
    }
  }
  PlanResult after;
  fits(result, p.budget_bytes, &after);
  st.peak_live_after = after.peak_live;
  st.arena_needed_after = after.arena_needed;
  g_in = std::move(result);
  if (stats) *stats = st;
  return LMS_OK;
}

}  // namespace lms
