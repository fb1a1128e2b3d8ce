"""Pins of the oracle's graph model and rewriter: the orders printed in Figures 2 and 3,
brute-force enumeration of valid control operations on small random graphs, hand-derived
chain cases, structural invariants of any rewrite, bit-identical evaluation of rewritten
graphs, and the lifetime rule of the peak-memory simulator."""
import itertools
import json
import os
import random

import numpy as np
import pytest

import workloads as W
from oracle import evaluate, model
from oracle.graph import Graph, READ, CONTROL, UPDATE, FWD, BWD
from oracle.rewrite import (Params, rewrite, direct_order, chain_rule, contract_swaps, peak_live_bytes, select)

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def by_name(g):
    return {n.name: n.id for n in g.nodes}


# ---------------------------------------------------------------- Section 3: orders
def test_fig1_expression_graph_orders():
    g = Graph()
    x, y, c, z = (g.add_variable(n) for n in ("x", "y", "5", "z"))
    plus = g.add_op("+", "add", [x, y])
    minus = g.add_op("-", "sub", [x, c])
    mul = g.add_op("*", "mul", [plus, minus])
    g.add_update_edge(mul, z)
    gam = g.gamma()
    assert [gam[v] for v in (x, y, c, z)] == [0, 0, 0, 0]
    assert gam[plus] == gam[minus] == 1 and gam[mul] == 2
    assert g.out(mul) == []                       # update edges lead to variables only
    assert g.reach(x) == {plus, minus, mul}


def test_fig2_orders():
    gold = json.load(open(os.path.join(GOLD, "fig2_orders.json")))
    # (a) x -> h -> f, f updates x
    g = Graph()
    x = g.add_variable("x")
    h = g.add_op("h", "op", [x])
    f = g.add_op("f", "op", [h])
    g.add_update_edge(f, x)
    gam = g.gamma()
    assert {n: gam[i] for n, i in by_name(g).items()} == gold["a"]
    # (b) f1 reads f and x
    f1 = g.add_op("f1", "op", [f, x])
    gam = g.gamma()
    assert {n: gam[i] for n, i in by_name(g).items()} == gold["b"]
    # (c) f2 reads f and updates x; a control edge f2 -> f1 pushes f1 one order later
    f2 = g.add_op("f2", "op", [f])
    g.add_update_edge(f2, x)
    assert g.gamma()[f1] == 3                     # without the control edge f1 and f2 are parallel
    g.add_control_edge(f2, f1)
    gam = g.gamma()
    assert {n: gam[i] for n, i in by_name(g).items()} == gold["c"]


def test_cycle_detected_and_no_control_into_variable():
    g = Graph()
    x = g.add_variable("x")
    a = g.add_op("a", "op", [x])
    b = g.add_op("b", "op", [a])
    g.add_control_edge(b, a)
    with pytest.raises(ValueError):
        g.gamma()
    with pytest.raises(AssertionError):
        g.add_control_edge(a, x)


# ---------------------------------------------------------------- Section 4: Figure 3
def fig3_graph():
    """A graph realising the orders of Figure 3: a chain c1..c24 below the variable gives
    order i to c_i; f1 = c10, f4 reads f1 (order 11), f3 reads f1 and c17 (order 18),
    f2 reads f1 and c24 (order 25); fj = c15, fi = c20."""
    g = Graph()
    x = g.add_variable("x", "input")
    prev, chain = x, {}
    for i in range(1, 25):
        prev = g.add_op(f"c{i}", "op", [prev], FWD)
        chain[i] = prev
    f1 = chain[10]
    f4 = g.add_op("f4", "op", [f1], FWD)
    f3 = g.add_op("f3", "op", [f1, chain[17]], FWD)
    f2 = g.add_op("f2", "op", [f1, chain[24]], FWD)
    return g, chain, f1, f2, f3, f4


def test_fig3_golden_rewrite():
    gold = json.load(open(os.path.join(GOLD, "fig3_rewrite.json")))
    g, chain, f1, f2, f3, f4 = fig3_graph()
    gam = g.gamma()
    assert {"f1": gam[f1], "f4": gam[f4], "f3": gam[f3], "f2": gam[f2]} == gold["orders_before"]
    # distances 15, 8 and 1 against alpha = 5; direct-order with distance 5 lands on orders 20 / 13,
    # the figure's f_i (20) is what distance 5 from f2 gives; f_j (15) is distance 3 from f3
    before = contract_swaps(g)
    p = Params(swap_branches=True, branch_threshold=5, ctrld_strategy="direct_order", lb=5, ub=10000,
               starting_op_names=["c10"], n_tensors=1)
    st = rewrite(g, p)
    assert (st.swap_outs, st.swap_ins, st.tensors) == (gold["swap_outs"], gold["swap_ins"], 1)
    so = [n for n in g.nodes if n.op == "swap_out"]
    assert len(so) == 1 and so[0].label == gold["swap_out_order"] and so[0].placement == "host"
    assert g.inputs(so[0].id) == [f1]
    si = {g.out(n.id)[0]: n for n in g.nodes if n.op == "swap_in"}
    assert set(si) == {f2, f3}
    assert f1 in g.inputs(f4)                                  # the short edge keeps reading f1
    assert f1 not in g.inputs(f2) and f1 not in g.inputs(f3)
    assert g.control_inputs(si[f2].id) == [chain[20]] and si[f2].label == gold["swap_in_order"]["f2"]
    # every vertex that existed before keeps its printed order
    assert contract_swaps(g) == before
    # f3's swap-in with the figure's control operation f_j (order 15): distance 3
    g2, chain2, f1b, f2b, f3b, _ = fig3_graph()
    assert direct_order(g2, g2.gamma(), f1b, f3b, 3, 10000) == chain2[15]
    st2 = rewrite(g2, Params(swap_branches=True, branch_threshold=5, ctrld_strategy="direct_order", lb=3,
                             starting_op_names=["c10"], n_tensors=1))
    si2 = {g2.out(n.id)[0]: n for n in g2.nodes if n.op == "swap_in"}
    assert si2[f3b].label == gold["swap_in_order"]["f3"] and g2.control_inputs(si2[f3b].id) == [chain2[15]]


# ---------------------------------------------------------------- Algorithms 1 and 2
def chain_net(depth, read_input=True):
    """x -> F1 -> ... -> Fd -> loss; backward B_d ... B_1 where B_i reads F_i's output, the
    gradient from B_{i+1} and (read_input) F_i's input tensor, the output of F_{i-1}."""
    g = Graph()
    x = g.add_variable("x", "input")
    F, prev = {}, x
    for i in range(1, depth + 1):
        w = g.add_variable(f"w{i}")
        F[i] = g.add_op(f"F{i}", "op", [prev, w], FWD)
        prev = F[i]
    loss = g.add_op("loss", "op", [prev], FWD)
    B, grad = {}, g.add_op("dloss", "op", [loss], BWD)
    for i in range(depth, 0, -1):
        ins = [grad, F[i]] + ([F[i - 1]] if (i > 1 and read_input) else [])
        B[i] = g.add_op(f"B{i}", "op", ins, BWD)
        grad = B[i]
    return g, F, B


@pytest.mark.parametrize("lb", [1, 2, 3])
def test_chain_rule_on_a_layer_chain(lb):
    # the gradient operation of layer i + lb triggers the swap-in of layer i's activation
    g, F, B = chain_net(8, read_input=False)
    gam = g.gamma()
    for i in range(1, 4):
        got = chain_rule(g, gam, F[i], B[i], lb, 10000)
        assert got == B[i + lb], (i, lb, g.nodes[got])
        assert gam[F[i]] < gam[got] < gam[B[i]] and B[i] in g.reach(got)
    # when B_j also reads F_{j-1}, F_{i+lb} has two backward readers, B_{i+lb} and B_{i+lb+1};
    # both are valid and the lowest id (B_{i+lb+1}, created first) is taken
    g, F, B = chain_net(8, read_input=True)
    gam = g.gamma()
    for i in range(1, 4):
        assert chain_rule(g, gam, F[i], B[i], lb, 10000) == B[i + lb + 1]


def test_strategy_null_cases():
    g, F, B = chain_net(5)
    gam = g.gamma()
    assert chain_rule(g, gam, F[1], B[1], 3, 2) is None          # lower bound above upper bound
    assert chain_rule(g, gam, F[1], B[1], 0, 0) is None          # upper bound zero
    assert chain_rule(g, gam, F[1], B[1], 50, 10000) is None     # forward phase exhausted first
    assert direct_order(g, gam, F[1], B[1], 1000, 10000) is None  # walks below f1
    assert direct_order(g, gam, F[1], B[1], 3, 2) is None         # empty range
    # direct-order with distance 1 is the operation right before f2
    d1 = direct_order(g, gam, F[1], B[1], 1, 10000)
    assert gam[d1] == gam[B[1]] - 1 and B[1] in g.reach(d1)


def random_dag(r, n_ops):
    g = Graph()
    g.add_variable("x", "input")
    g.add_variable("w")
    for i in range(n_ops):
        k = r.randint(1, min(3, len(g.nodes)))
        ins = r.sample(range(len(g.nodes)), k)
        # phases non-decreasing along the id order so forward never reads backward
        phase = FWD if i < n_ops * 0.55 else BWD
        g.add_op(f"n{i}", "op", ins, phase)
    return g


def test_strategies_against_brute_force_on_random_dags():
    r = random.Random(1807)
    checked_dir = checked_chain = nulls = 0
    for trial in range(300):
        g = random_dag(r, r.randint(5, 10))
        gam = g.gamma()
        ops = [n.id for n in g.nodes if not n.is_var]
        for f1, f2 in itertools.permutations(ops, 2):
            if f2 not in g.readers(f1) or gam[f2] - gam[f1] <= 1:
                continue
            valid = {v for v in ops if gam[f1] < gam[v] < gam[f2] and f2 in g.reach(v)}
            for lb in (1, 2):
                d = direct_order(g, gam, f1, f2, lb, 10000)
                # brute force: the largest order k <= gamma(f2) - lb, k > gamma(f1), holding a valid vertex
                ks = [gam[v] for v in valid if gam[v] <= gam[f2] - lb]
                if ks:
                    assert d in valid and gam[d] == max(ks)
                    checked_dir += 1
                else:
                    assert d is None
                    nulls += 1
                c = chain_rule(g, gam, f1, f2, lb, 10000)
                if c is not None:
                    assert c in valid and g.nodes[c].phase == BWD
                    # c reads a forward operation at least lb forward steps below f1
                    fw_parents = [u for u in g.inputs(c) if g.nodes[u].phase == FWD and not g.nodes[u].is_var]
                    # (some forward path of that length exists; the walk may meet a vertex at several levels)
                    assert any(max(_fwd_path_lengths(g, f1, u), default=-1) >= lb for u in fw_parents)
                    checked_chain += 1
                else:
                    # brute force: no valid backward vertex hangs off any forward vertex at depth >= lb
                    for u in ops:
                        dep = _fwd_depth(g, f1, u)
                        if dep is None or dep < lb or g.nodes[u].phase != FWD:
                            continue
                        assert not [b for b in g.out(u) if b in valid and g.nodes[b].phase == BWD]
    assert checked_dir > 200 and checked_chain > 50 and nulls > 5


def _fwd_path_lengths(g, f1, u):
    """Lengths of all paths f1 -> u whose vertices after f1 are forward operations."""
    if f1 == u:
        return {0}
    out = set()
    for v in g.out(f1):
        if g.nodes[v].phase == FWD and not g.nodes[v].is_var:
            out |= {l + 1 for l in _fwd_path_lengths(g, v, u)}
    return out


def _fwd_depth(g, f1, u):
    """Breadth-first depth of u below f1 through forward operations only."""
    level, seen, d = [f1], {f1}, 0
    while level:
        if u in level:
            return d
        nxt = []
        for s in level:
            for v in g.out(s):
                if v not in seen and g.nodes[v].phase == FWD and not g.nodes[v].is_var:
                    seen.add(v)
                    nxt.append(v)
        level, d = nxt, d + 1
    return None


# ---------------------------------------------------------------- invariants of a rewrite
PARAM_SETS = [
    Params(), Params(lb=2), Params(ctrld_strategy="direct_order"), Params(ctrld_strategy="direct_order", lb=3),
    Params(fuse_swapins=True), Params(n_tensors=2), Params(swap_branches=True, branch_threshold=2),
    Params(swap_branches=True, branch_threshold=0, fuse_swapins=True, lb=2), Params(fuse_swapins=True, fuse_distance=1),
    Params(excl_types=["relu"]), Params(incl_types=["relu"]), Params(excl_scopes=["conv2"]),
]
SPECS = {
    "chain": lambda: W.tiny_chain(batch=2, size=6, width=4, depth=4, classes=3),
    "stage": lambda: W.bottleneck_stage(batch=1, size=4, cin=8, width=4, blocks=2),
    "resnet": lambda: W.resnet50(batch=1, size=16, classes=4, stage_blocks=(1, 1), base=4),
    "unet": lambda: W.unet3d(batch=1, size=4, base=2, levels=2, classes=3),
}


def check_valid(g0, g1, st):
    gam0 = g0.gamma()
    gam1 = g1.gamma()                                           # raises on a cycle
    assert contract_swaps(g1) == contract_swaps(g0)
    sos = [n for n in g1.nodes if n.op == "swap_out"]
    sis = [n for n in g1.nodes if n.op == "swap_in"]
    assert (len(sos), len(sis)) == (st.swap_outs, st.swap_ins)
    assert len({g1.inputs(s.id)[0] for s in sos}) == len(sos)   # swap-outs are fused: one per tensor
    for s in sos:
        u = g1.inputs(s.id)[0]
        assert not g1.nodes[u].is_var and g1.nodes[u].phase == FWD and s.label == gam0[u] + 1
        assert s.placement == "host"
    for s in sis:
        assert len(g1.inputs(s.id)) == 1 and g1.nodes[g1.inputs(s.id)[0]].op == "swap_out"
        ctl = g1.control_inputs(s.id)
        assert len(ctl) == 1
        so = g1.inputs(s.id)[0]
        u = g1.inputs(so)[0]
        for v in g1.out(s.id):
            # Section 4.3: gamma(swap-out) < gamma(control op) < gamma(consumer), with printed labels
            assert gam0[u] < gam0[ctl[0]] < gam0[v]
        assert s.label == gam0[ctl[0]] + 1
    for e in g1.edges:                                          # variable edges are never rewritten
        if g1.nodes[e.src].is_var or g1.nodes[e.dst].is_var:
            assert g1.nodes[e.src].op not in ("swap_in", "swap_out")
            assert g1.nodes[e.dst].op not in ("swap_in", "swap_out")
        if e.action == CONTROL:
            assert not g1.nodes[e.dst].is_var


@pytest.mark.parametrize("sname", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAM_SETS)))
def test_rewrite_is_valid_and_changes_no_value(sname, pi):
    spec = SPECS[sname]()
    g0, ids = model.build(spec)
    g1 = g0.copy()
    st = rewrite(g1, PARAM_SETS[pi])
    check_valid(g0, g1, st)
    if PARAM_SETS[pi].fuse_swapins and PARAM_SETS[pi].fuse_distance > 1000:
        assert st.swap_ins == st.swap_outs            # one swap-out and one swap-in per tensor
    else:
        assert st.swap_ins >= st.swap_outs
    t = W.make_tensors(spec, affine="random")
    a = evaluate.run(g0, t)
    b = evaluate.run(g1, t)
    for name, v in ids.items():
        assert np.array_equal(np.asarray(a[v]), np.asarray(b[v])), name


def test_default_rewrite_swaps_every_forward_to_backward_tensor():
    spec = SPECS["chain"]()
    g0, ids = model.build(spec)
    gam = g0.gamma()
    expect = set()
    for e in g0.edges:
        u, v = g0.nodes[e.src], g0.nodes[e.dst]
        if e.action == READ and not u.is_var and u.phase == FWD and v.phase == BWD and gam[v.id] - gam[u.id] > 1:
            expect.add(u.id)
    g1 = g0.copy()
    st = rewrite(g1, Params())
    assert set(st.swapped) == expect and st.tensors == len(expect) >= 5
    # breadth-first order from the input: selection order follows depth
    assert st.swapped == sorted(st.swapped, key=lambda u: gam[u])
    g2 = g0.copy()
    st2 = rewrite(g2, Params(n_tensors=3))
    assert st2.swapped == st.swapped[:3]
    g3 = g0.copy()
    assert rewrite(g3, Params(n_tensors=0)).tensors == 0 and len(g3.nodes) == len(g0.nodes)


def test_unfused_swapins_one_per_consumer():
    spec = SPECS["stage"]()
    g0, _ = model.build(spec)
    g1, g2 = g0.copy(), g0.copy()
    s1 = rewrite(g1, Params())
    s2 = rewrite(g2, Params(fuse_swapins=True))
    assert s1.swap_outs == s2.swap_outs == s2.swap_ins
    assert s1.swap_ins > s1.swap_outs                  # some tensor has several backward readers
    assert s1.swap_outs + s1.swap_ins > 2 * s1.tensors == s2.swap_outs + s2.swap_ins


# ---------------------------------------------------------------- Section 3.5: lifetimes
def test_peak_simulator_lifetime_rule():
    g = Graph()
    x = g.add_variable("x", "input")
    a = g.add_op("a", "op", [x])
    b = g.add_op("b", "op", [a])
    c = g.add_op("c", "op", [b])
    d = g.add_op("d", "op", [c, a])       # a lives until d: lifetime gamma(d) - gamma(a) = 3
    gam = g.gamma()
    assert gam[d] - gam[a] == 3
    nbytes = {x: 1000, a: 10, b: 20, c: 40, d: 80}
    peak, trace = peak_live_bytes(g, [x, a, b, c, d], nbytes)
    # a | a+b | a+c (b freed after c ran; c is allocated while b is still live) | a+c+d
    assert trace == [0, 10, 30, 70, 130] and peak == 130
    # swapping a out right after b and back in before d removes it from the middle of the run
    so = g.add_op("so", "swap_out", [a])
    si = g.add_op("si", "swap_in", [so])
    for e in g.edges:
        if e.src == a and e.dst == d:
            e.src = si
    nbytes[so] = nbytes[si] = 10
    peak2, trace2 = peak_live_bytes(g, [x, a, b, so, c, si, d], nbytes)
    assert trace2 == [0, 10, 30, 30, 60, 50, 130]


def test_rewriting_lowers_simulated_peak_on_a_chain():
    spec = W.tiny_chain(batch=2, size=8, width=8, depth=6)
    g0, ids = model.build(spec)
    t = W.make_tensors(spec)
    vals = evaluate.run(g0, t)
    g1 = g0.copy()
    rewrite(g1, Params())
    vals1 = evaluate.run(g1, t)

    def order_and_bytes(g, vals):
        gam = g.gamma()
        order = sorted((n.id for n in g.nodes), key=lambda v: (gam[v], v))
        return order, {v: np.asarray(vals[v]).size * 2 for v in order}
    p0, _ = peak_live_bytes(g0, *order_and_bytes(g0, vals))
    p1, _ = peak_live_bytes(g1, *order_and_bytes(g1, vals1))
    assert p1 < p0
