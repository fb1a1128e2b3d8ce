"""Swap-out / swap-in graph rewriting, step by step as the paper states it.

TEST INFRASTRUCTURE ONLY; nothing in the product path may import it.

Section 4: swap-out insertion (Eq. 1-2), introduction of swap-ins (Eq. 3-5),
fusing of swap-outs (4.2.2) and swap-ins (4.2.3), and the two strategies that
pick the control operation of a swap-in (Algorithm 1 direct-order,
Algorithm 2 chain-rule).  Section 5.1 and Table 2: which edges are rewritten
and the parameters.  Readings taken where the text is silent or ambiguous:

* orders gamma are minimal levels (graph.Graph.gamma); the orders of vertices
  that existed before rewriting are not recomputed, an inserted swap-out gets
  gamma(producer)+1 and a swap-in gets gamma(control op)+1 (Figure 3);
* the breadth-first walk starts at the variables of kind "input" (or at
  starting_op_names), visits forward operations level by level, each level in
  ascending vertex id, and n_tensors counts tensors;
* an edge (u, v) qualifies only if gamma(v) - gamma(u) > 1 (no operation can
  sit between closer ones, Section 4.1), forward-to-forward edges additionally
  need swap_branches and gamma(v) - gamma(u) > branch_threshold (Section 5.1);
* GET takes the lowest vertex id; both searches run on the graph as it was
  before any rewriting; "f2 reachable from f" is transitive reachability in
  both algorithms;
* when a strategy returns nothing, the direct-order walk is repeated from
  distance 1 without the reachability filter; if that fails too the edge is
  left as it was;
* fused swap-ins: consumers whose order is within fuse_distance of the
  earliest consumer of their group share one swap-in (default: all of them).
"""
from dataclasses import dataclass, field
from typing import Optional, Sequence

from .graph import Graph, Edge, Node, READ, CONTROL, UPDATE, FWD, BWD, SWAP

INF = 1 << 60


@dataclass
class Params:
    """Table 2.  optimizer_scopes is represented by the per-vertex phase tag."""
    n_tensors: int = -1
    lb: int = 1
    ub: int = 10000
    ctrld_strategy: str = "chain_rule"
    fuse_swapins: bool = False
    fuse_distance: int = INF
    swap_branches: bool = False
    branch_threshold: int = 0
    starting_op_names: Optional[Sequence[str]] = None
    starting_scope: Optional[str] = None
    excl_scopes: Sequence[str] = ()
    incl_scopes: Sequence[str] = ()
    excl_types: Sequence[str] = ()
    incl_types: Sequence[str] = ()
    # Recomputation (named as future work in Section 7 of the paper, after the related work it cites in Section 2):
    # a tensor that would be swapped and whose producer is one of these cheap operations is produced a second time
    # next to its late consumers instead of travelling to the host and back.
    recompute: bool = False
    cheap_ops: Sequence[str] = ("maxpool", "concat", "gap")
    # Chained recomputation (same future work; the paper gives no rule, this one is the library's own): tensors the
    # selection would swap are recomputed next to their late consumers from the tensors that stay stored, a
    # recomputed tensor possibly feeding the recomputation of the next, up to recompute_depth tensors in a row.
    # recompute_ops: operation kinds that may be recomputed (empty = pass off); recompute_set: the producers to
    # recompute, given explicitly (then the depth rule is not applied).
    recompute_ops: Sequence[str] = ()
    recompute_depth: int = 0
    recompute_set: Optional[Sequence[int]] = None


@dataclass
class Stats:
    tensors: int = 0
    swap_outs: int = 0
    swap_ins: int = 0
    control_edges: int = 0
    unrewritten: int = 0
    recomputed: int = 0                               # copies of cheap operations inserted
    swapped: list = field(default_factory=list)      # producer ids, in selection order


def direct_order(g: Graph, gam, f1, f2, lo, hi, need_reach=True):
    """Algorithm 1: walk back from f2 one order at a time."""
    low = max(gam[f2] - hi + 1, gam[f1])
    for i in range(lo, hi + 1):
        k = gam[f2] - i
        if k <= low:
            return None
        cand = [n.id for n in g.nodes if not n.is_var and gam[n.id] == k]
        if need_reach:
            cand = [f for f in cand if f2 in g.reach(f)]
        if cand:
            return min(cand)
    return None


def chain_rule(g: Graph, gam, f1, f2, lo, hi):
    """Algorithm 2: level-by-level walk down the forward phase from f1; inside the
    [lo, hi] window, a backward consumer of the current forward operation that lies
    strictly between f1 and f2 in order and reaches f2 is the control operation."""
    s1, s2, closed = [f1], [], set()
    while s1:
        if hi == 0 or lo > hi:
            return None
        s = min(s1)
        s1.remove(s)
        outs = g.out(s)
        if lo <= 0:
            b = [f for f in outs if g.nodes[f].phase == BWD and gam[f1] < gam[f] < gam[f2]
                 and f2 in g.reach(f)]
            if b:
                return min(b)
        for f in outs:
            if g.nodes[f].phase != FWD or g.nodes[f].is_var:
                continue
            if f in closed:
                continue
            if f not in s2:
                s2.append(f)
        closed.add(s)
        if not s1:
            lo, hi = lo - 1, hi - 1
            s1, s2 = s2, []
    return None


def _type_scope_ok(node: Node, p: Params):
    scope_hit = lambda scopes: any(node.name.startswith(s) for s in scopes)
    if p.incl_types and node.op not in p.incl_types:
        return False
    if p.incl_scopes and not scope_hit(p.incl_scopes):
        return False
    if node.op in p.excl_types or scope_hit(p.excl_scopes):
        return False
    return True


def select(g: Graph, gam, p: Params):
    """Tensors to swap, in breadth-first order: [(producer, [qualifying consumers])]."""
    if p.starting_op_names:
        level = sorted(n.id for n in g.nodes if n.name in p.starting_op_names)
    elif p.starting_scope:
        level = sorted(n.id for n in g.nodes if n.name.startswith(p.starting_scope))
    else:
        level = sorted(n.id for n in g.nodes if n.is_var and n.kind == "input")
        if not level:
            level = sorted(n.id for n in g.nodes if n.is_var)
    seen = set(level)
    picked = []
    while level:
        nxt = []
        for u in level:
            nu = g.nodes[u]
            if not nu.is_var and nu.phase == FWD and _type_scope_ok(nu, p):
                cons = []
                for v in g.readers(u):
                    nv = g.nodes[v]
                    d = gam[v] - gam[u]
                    if nv.is_var or d <= 1:
                        continue
                    if nv.phase == BWD or (p.swap_branches and nv.phase == FWD and d > p.branch_threshold):
                        cons.append(v)
                if cons:
                    picked.append((u, cons))
                    if p.n_tensors >= 0 and len(picked) >= p.n_tensors:
                        return picked[:max(p.n_tensors, 0)]
            for v in g.readers(u):
                nv = g.nodes[v]
                if v not in seen and not nv.is_var and nv.phase == FWD:
                    seen.add(v)
                    nxt.append(v)
        level = sorted(nxt)
    return picked if p.n_tensors < 0 else picked[:p.n_tensors]


def _consumer_groups(orig: Graph, gam, u, cons, p: Params, st: Stats):
    """Consumers of u's tensor grouped for one late copy each (Section 4.2.3) with the control operation that
    triggers the copy (Section 4.3): [(consumers, control op)]."""
    cons = sorted(cons, key=lambda v: (gam[v], v))
    if p.fuse_swapins:
        groups = []
        for v in cons:
            if groups and gam[v] - gam[groups[-1][0]] <= p.fuse_distance:
                groups[-1].append(v)
            else:
                groups.append([v])
    else:
        groups = [[v] for v in cons]
    plans = []
    for grp in groups:
        f2 = grp[0]
        if p.ctrld_strategy == "chain_rule":
            ctl = chain_rule(orig, gam, u, f2, p.lb, p.ub)
        elif p.ctrld_strategy == "direct_order":
            ctl = direct_order(orig, gam, u, f2, p.lb, p.ub)
        else:
            raise ValueError(p.ctrld_strategy)
        if ctl is None:
            ctl = direct_order(orig, gam, u, f2, 1, p.ub, need_reach=False)
        if ctl is None:
            st.unrewritten += len(grp)
            continue
        plans.append((grp, ctl))
    return plans


def recompute_cheap(g: Graph, p: Params, st: Stats):
    """Pass that runs before the swaps are inserted: every tensor the selection of Section 5.1 would swap (whatever
    n_tensors says) whose producer is a cheap operation gets, per group of late consumers, a copy of the producer
    with the same inputs, triggered by a control edge exactly as a swap-in would be; the consumers read the copy.
    The copy carries the phase of its first consumer, so in the swap pass that follows its inputs count as tensors
    with a late consumer like any other."""
    gam = g.gamma()
    orig = g.copy()
    everything = Params(**{**p.__dict__, "n_tensors": -1})
    for u, cons in select(orig, gam, everything):
        nu = orig.nodes[u]
        if nu.op not in p.cheap_ops:
            continue
        for grp, ctl in _consumer_groups(orig, gam, u, cons, p, st):
            c = g.add_op(f"{nu.name}/recompute{grp[0]}", nu.op, orig.inputs(u), phase=orig.nodes[grp[0]].phase, attrs=nu.attrs)
            g.nodes[c].label = gam[ctl] + 1
            for e in g.edges:
                if e.action == READ and e.src == u and e.dst in grp:
                    e.src = c
            g.add_control_edge(ctl, c)
            st.recomputed += 1
            st.control_edges += 1


def _control_for(orig: Graph, gam, u, f2, p: Params):
    """Control operation that triggers a late copy of u's tensor ahead of consumer f2 (Section 4.3), or None."""
    if p.ctrld_strategy == "chain_rule":
        ctl = chain_rule(orig, gam, u, f2, p.lb, p.ub)
    elif p.ctrld_strategy == "direct_order":
        ctl = direct_order(orig, gam, u, f2, p.lb, p.ub)
    else:
        raise ValueError(p.ctrld_strategy)
    if ctl is None:
        ctl = direct_order(orig, gam, u, f2, 1, p.ub, need_reach=False)
    return ctl


def recompute_by_depth(g: Graph, picked, p: Params):
    """The depth rule: walking the selected tensors in creation order, a tensor is recomputed if its producer is of a
    kind in recompute_ops and the chain of recomputed tensors that ends in it stays within recompute_depth; every
    other tensor counts as stored (chain length 0).  Returns the producers to recompute."""
    depth, chosen = {}, []
    cand = {u for u, _ in picked}
    for u in sorted(cand):
        if g.nodes[u].op not in p.recompute_ops:
            continue
        d = 1 + max((depth.get(i, 0) for i in g.inputs(u) if not g.nodes[i].is_var), default=0)
        if d <= p.recompute_depth:
            depth[u] = d
            chosen.append(u)
    return chosen


def recompute_chained(g: Graph, p: Params, st: Stats):
    """Pass that runs before the swaps are inserted.  Every chosen tensor gets ONE late copy of its producer, read
    by all its late consumers (the consumers the selection of Section 5.1 names).  A copy reads the copies of those
    of its inputs that are recomputed too, and the stored tensors themselves otherwise (the swap pass that follows
    sees those as tensors with a late consumer).  The copy of u is triggered by a control edge from the operation
    the strategy of Section 4.3 picks for (u, t), t being the earliest late consumer that u serves directly or
    through copies that read it; a copy that feeds another copy is never triggered later (in creation order of
    the control operations) than the copy it feeds: it then takes that copy's control operation.  Copies are
    created in the creation order of their originals, so a chain executes front to back."""
    gam = g.gamma()
    orig = g.copy()
    everything = Params(**{**p.__dict__, "n_tensors": -1})
    picked = select(orig, gam, everything)
    cons_of = dict(picked)
    chosen = list(p.recompute_set) if p.recompute_set is not None else recompute_by_depth(orig, picked, p)
    # A tensor given explicitly need not have a late consumer of its own: a forward tensor that only a recomputed
    # producer reads (the shortcut branch of a residual sum, say) is then recomputed for that copy alone.
    chosen = sorted(u for u in set(chosen) if u in cons_of or (not orig.nodes[u].is_var and orig.nodes[u].phase == FWD))
    key = lambda v: (gam[v], v)
    target, ctrl, feeds = {}, {}, {}
    for u in reversed(chosen):
        # late consumers u serves: its own, and (through their copies) those of the chosen tensors that read u
        served = [min(cons_of[u], key=key)] if u in cons_of else []
        for w in feeds.get(u, ()):
            if w in ctrl:
                served.append(target[w])
        if not served:
            continue                       # nothing late reads it, directly or through a copy
        t = min(served, key=key)
        ctl = _control_for(orig, gam, u, t, p)
        if ctl is None:
            st.unrewritten += len(cons_of.get(u, ()))
            continue
        for w in feeds.get(u, ()):
            if w in ctrl and ctrl[w] < ctl:
                ctl = ctrl[w]
        target[u], ctrl[u] = t, ctl
        for i in orig.inputs(u):
            if i in chosen:
                feeds.setdefault(i, []).append(u)
    copy = {}
    for u in chosen:
        if u not in ctrl:
            continue
        nu = orig.nodes[u]
        ins = [copy.get(i, i) for i in orig.inputs(u)]
        c = g.add_op(f"{nu.name}/recompute", nu.op, ins, phase=orig.nodes[target[u]].phase, attrs=nu.attrs)
        g.nodes[c].label = max([gam[ctrl[u]] + 1] + [g.nodes[i].label + 1 for i in ins if i in copy.values()])
        for e in g.edges:
            if e.action == READ and e.src == u and e.dst in cons_of.get(u, ()):
                e.src = c
        g.add_control_edge(ctrl[u], c)
        copy[u] = c
        st.recomputed += 1
        st.control_edges += 1
    return copy


def rewrite(g: Graph, p: Params = Params()):
    """Rewrites g in place; returns Stats.  Orders of inserted vertices are left in Node.label."""
    st = Stats()
    if p.recompute:
        recompute_cheap(g, p, st)
    elif p.recompute_ops and (p.recompute_depth > 0 or p.recompute_set is not None):
        recompute_chained(g, p, st)
    gam = g.gamma()
    orig = g.copy()
    if p.n_tensors == 0:
        return st
    for u, cons in select(orig, gam, p):
        plans = _consumer_groups(orig, gam, u, cons, p, st)
        if not plans:
            continue
        so = g.add_op(f"{g.nodes[u].name}/swap_out", "swap_out", [u], phase=SWAP)
        g.nodes[so].placement = "host"
        g.nodes[so].label = gam[u] + 1
        st.swap_outs += 1
        st.tensors += 1
        st.swapped.append(u)
        for grp, ctl in plans:
            si = g.add_op(f"{g.nodes[u].name}/swap_in{grp[0]}", "swap_in", [so], phase=SWAP)
            g.nodes[si].placement = "host"
            g.nodes[si].label = gam[ctl] + 1
            for e in g.edges:
                if e.action == READ and e.src == u and e.dst in grp:
                    e.src = si
            g.add_control_edge(ctl, si)
            st.swap_ins += 1
            st.control_edges += 1
    return st


def contract_swaps(g: Graph):
    """Edge multiset of g with every swap-out / swap-in pair contracted back into the
    direct edge it replaced (Eq. 2 and Eq. 5 read right to left) and the control
    edges into swap-ins dropped."""
    def origin(v):
        while g.nodes[v].op in ("swap_in", "swap_out"):
            v = g.inputs(v)[0]
        return v
    keys = []
    for e in g.edges:
        if g.nodes[e.dst].op in ("swap_in", "swap_out"):
            continue
        keys.append((origin(e.src) if e.action == READ else e.src, e.dst, e.action, e.slot))
    return sorted(keys)


def peak_live_bytes(g: Graph, order, nbytes):
    """Largest sum of device-resident tensor bytes over a sequential run in `order`.

    Lifetime rule of Section 3.5: a tensor lives from the operation producing it to the
    last operation consuming it.  Variables and host-placed tensors (swap-out outputs)
    do not count; a swap-in output is a new device tensor.  Returns (peak, per-step list)."""
    pos = {v: i for i, v in enumerate(order)}
    last = {}
    for e in g.edges:
        if e.action == READ and e.dst in pos and e.src in pos:
            last[e.src] = max(last.get(e.src, pos[e.src]), pos[e.dst])
    live, peak, trace = 0, 0, []
    dying = {}
    for i, v in enumerate(order):
        n = g.nodes[v]
        on_device = not n.is_var and n.op != "swap_out"
        if on_device:
            live += nbytes[v]
            dying.setdefault(last.get(v, i), []).append(v)
        peak = max(peak, live)
        trace.append(live)
        for d in dying.pop(i, ()):
            live -= nbytes[d]
    return peak, trace
