"""Pins of the oracle's chained recomputation pass (recompute_chained): which tensors the depth rule picks on a
hand-checked chain, the structure of the copies (one per tensor, chained, triggered in order), unchanged values of
every original vertex whatever swap pass follows, and the memory effect."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate, model
from oracle.graph import Graph, FWD, BWD
from oracle.rewrite import Params, rewrite, select, recompute_by_depth, peak_live_bytes

SPECS = {
    "chain": lambda: W.tiny_chain(batch=1, size=8, width=4, depth=4, classes=3),
    "pool_net": lambda: W.pool_net(),
    "updown_net": lambda: W.updown_net(),
    "unet": lambda: W.unet3d(batch=1, size=8, base=4, levels=3, classes=3),
    "resnet": lambda: W.resnet50(batch=1, size=16, classes=4, stage_blocks=(2, 1), base=4),
}
ALL_OPS = ("conv", "affine", "bias", "add", "relu", "maxpool", "gap", "tconv", "concat")
PARAMS = [Params(recompute_ops=ALL_OPS, recompute_depth=1), Params(recompute_ops=ALL_OPS, recompute_depth=2, fuse_swapins=True),
          Params(recompute_ops=ALL_OPS, recompute_depth=3, ctrld_strategy="direct_order", lb=2),
          Params(recompute_ops=ALL_OPS, recompute_depth=50, fuse_swapins=True, n_tensors=0),
          Params(recompute_ops=("conv", "relu"), recompute_depth=4, swap_branches=True, branch_threshold=2, fuse_swapins=True),
          Params(recompute_ops=ALL_OPS, recompute_depth=2, n_tensors=3)]


def layer_chain(n_layers):
    """x -> f1 -> ... -> fn -> loss with backward operations b_n .. b_1; b_i reads f_i's output and the gradient
    from b_{i+1}: the smallest graph in which every forward tensor has one late consumer."""
    g = Graph()
    x = g.add_variable("x", "input")
    f, cur = [], x
    for i in range(n_layers):
        cur = g.add_op(f"f{i + 1}", "layer", [cur], FWD)
        f.append(cur)
    loss = g.add_op("loss", "loss", [cur], FWD)
    grad = g.add_op("dloss", "loss_bwd", [loss], BWD)
    b = {}
    for i in range(n_layers - 1, -1, -1):
        grad = g.add_op(f"b{i + 1}", "layer_bwd", [grad, f[i]], BWD)
        b[i] = grad
    return g, f, b


def test_depth_rule_on_a_hand_checked_chain():
    g, f, b = layer_chain(6)
    gam = g.gamma()
    picked = select(g, gam, Params())
    assert [u for u, _ in picked] == f                # f6 too: b6 lies three orders after it (loss, dloss in between)
    p = lambda d: Params(recompute_ops=("layer",), recompute_depth=d)
    names = lambda ids: [g.nodes[u].name for u in ids]
    # depth 1: a recomputed tensor may only read stored tensors -> every other one, starting at the input
    assert names(recompute_by_depth(g, picked, p(1))) == ["f1", "f3", "f5"]
    # depth 2: two in a row, then one stored
    assert names(recompute_by_depth(g, picked, p(2))) == ["f1", "f2", "f4", "f5"]
    assert names(recompute_by_depth(g, picked, p(0))) == []
    assert names(recompute_by_depth(g, picked, p(9))) == names(f)


def test_chain_copies_by_hand():
    """6-layer chain, depth 2, chain-rule with lb = 1.  f1 and f2 are recomputed, f3 stored, f4 and f5 recomputed, f6 stored.
    Late consumer of f_i is b_i; the chain-rule control operation of (f_i, b_i) is the backward operation of the
    next layer, b_{i+1}.  f4 feeds the copy of f5, which b6 triggers, so the copy of f4 serves b5 first (through
    f5's copy) and is triggered by b6 as well, not by its own b5."""
    g, f, b = layer_chain(6)
    g1 = g.copy()
    st = rewrite(g1, Params(recompute_ops=("layer",), recompute_depth=2, n_tensors=0))
    assert st.recomputed == 4 and st.control_edges == 4 and st.swap_outs == 0
    c = {n.name: n.id for n in g1.nodes}
    for name in ("f1", "f2", "f4", "f5"):
        assert f"{name}/recompute" in c
    assert "f3/recompute" not in c
    ins = lambda name: g1.inputs(c[name])
    assert ins("f1/recompute") == [c["x"]]
    assert ins("f2/recompute") == [c["f1/recompute"]]
    assert ins("f4/recompute") == [c["f3"]]                       # the stored tensor itself
    assert ins("f5/recompute") == [c["f4/recompute"]]
    assert g1.control_inputs(c["f5/recompute"]) == [c["b6"]]
    assert g1.control_inputs(c["f4/recompute"]) == [c["b6"]]
    assert g1.control_inputs(c["f2/recompute"]) == [c["b3"]]
    assert g1.control_inputs(c["f1/recompute"]) == [c["b3"]]
    # the backward operations read the copies, the forward chain still reads the originals
    assert g1.inputs(c["b5"])[1] == c["f5/recompute"] and g1.inputs(c["b4"])[1] == c["f4/recompute"]
    assert g1.inputs(c["b3"])[1] == c["f3"] and g1.inputs(c["f6"]) == [c["f5"]]
    gam0, gam1 = g.gamma(), g1.gamma()
    assert g1.nodes[c["f4/recompute"]].label == gam0[c["b6"]] + 1
    assert g1.nodes[c["f5/recompute"]].label == gam0[c["b6"]] + 2
    assert gam1[c["f4/recompute"]] < gam1[c["f5/recompute"]] < gam1[c["b5"]]
    # lifetimes: with 2-byte tensors of equal size the peak of live tensors drops from 6 forward tensors
    # (+ the gradient) to the stored one plus what one segment needs
    nbytes0 = {n.id: 1 for n in g.nodes if not n.is_var}
    nbytes1 = {n.id: 1 for n in g1.nodes if not n.is_var}
    o0 = sorted((n.id for n in g.nodes if not n.is_var), key=lambda v: (gam0[v], v))
    o1 = sorted((n.id for n in g1.nodes if not n.is_var), key=lambda v: (gam1[v], v))
    p0, p1 = peak_live_bytes(g, o0, nbytes0)[0], peak_live_bytes(g1, o1, nbytes1)[0]
    assert p1 < p0


@pytest.mark.parametrize("sname", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_chained_copies_are_valid_and_change_no_value(sname, pi):
    spec = SPECS[sname]()
    p = PARAMS[pi]
    g0, ids = model.build(spec)
    g1 = g0.copy()
    st = rewrite(g1, p)
    gam0 = g0.gamma()
    gam1 = g1.gamma()                                                # acyclic
    n0 = len(g0.nodes)
    by_name = {n.name: n for n in g0.nodes}
    copies = [n for n in g1.nodes[n0:] if n.name.endswith("/recompute")]
    assert len(copies) == st.recomputed
    assert len({n.name for n in copies}) == len(copies)             # one copy per tensor
    copy_of = {by_name[c.name[:-len("/recompute")]].id: c.id for c in copies}
    everything = Params(**{**p.__dict__, "n_tensors": -1, "recompute_depth": 0, "recompute_ops": ()})
    cons_of = dict(select(g0, gam0, everything))
    restored = lambda v: g1.inputs(g1.inputs(v)[0])[0] if g1.nodes[v].op == "swap_in" else v
    for u, cid in copy_of.items():
        src, c = g0.nodes[u], g1.nodes[cid]
        assert c.op == src.op and c.attrs == src.attrs and src.phase == FWD and src.op in p.recompute_ops
        for a, b in zip(g0.inputs(u), g1.inputs(cid)):
            b = restored(b)
            assert b == copy_of.get(a, a), (src.name, a, b)            # the copy of a recomputed input, else the input itself
        (ctl,) = g1.control_inputs(cid)
        assert ctl < n0 and gam0[u] < gam0[ctl]
        # every late consumer of the original now reads the copy, and runs after it
        for v in cons_of[u]:
            assert cid in [restored(i) for i in g1.inputs(v)] and u not in g1.inputs(v)
            assert gam1[cid] < gam1[v] and gam0[ctl] < gam0[v]
        # a copy that feeds another copy is triggered no later than that copy
        for v in g1.readers(cid):
            if v in copy_of.values():
                (ctl_v,) = g1.control_inputs(v)
                assert ctl <= ctl_v and gam1[cid] < gam1[v]
    # chains respect the depth limit
    depth = {}
    for u in sorted(copy_of):
        depth[u] = 1 + max((depth.get(i, 0) for i in g0.inputs(u)), default=0)
        assert depth[u] <= p.recompute_depth
    # values: every original vertex evaluates to the same bits, with the swap pass applied on top
    t = W.make_tensors(spec, affine="random")
    a = evaluate.run(g0, t)
    b = evaluate.run(g1, t)
    for name, v in ids.items():
        assert np.array_equal(np.asarray(a[v]), np.asarray(b[v])), name
    for u, cid in copy_of.items():
        assert np.array_equal(np.asarray(a[u]), np.asarray(b[cid]))


def test_recomputed_tensors_are_not_swapped_and_fewer_bytes_cross():
    spec = SPECS["resnet"]()
    g0, ids = model.build(spec)
    t = W.make_tensors(spec)
    vals = evaluate.run(g0, t)
    size = lambda v: int(np.asarray(vals[v]).size)
    g_swap, g_rec = g0.copy(), g0.copy()
    s_swap = rewrite(g_swap, Params(fuse_swapins=True))
    s_rec = rewrite(g_rec, Params(fuse_swapins=True, recompute_ops=ALL_OPS, recompute_depth=3))
    assert s_rec.recomputed > 0
    recomputed = {n.name[:-len("/recompute")] for n in g_rec.nodes if n.name.endswith("/recompute")}
    swapped_names = {g0.nodes[u].name for u in s_rec.swapped if u < len(g0.nodes)}
    assert not (recomputed & swapped_names)
    assert sum(size(u) for u in s_rec.swapped if u < len(g0.nodes)) < sum(size(u) for u in s_swap.swapped)


def forward_only_ancestors(g, cons_of, u):
    """u and the forward tensors behind it that no late operation reads, up to the first stored (late-read) ones."""
    out, todo = [], [u]
    while todo:
        v = todo.pop()
        out.append(v)
        for i in g.inputs(v):
            n = g.nodes[i]
            if not n.is_var and n.phase == FWD and i not in cons_of and i not in out:
                todo.append(i)
    return sorted(set(out))


@pytest.mark.parametrize("sname", ["resnet", "unet", "updown_net"])
def test_explicit_set_recomputes_forward_only_tensors_for_the_copies_that_read_them(sname):
    """Tensors named explicitly: a forward tensor without a late consumer of its own (an affine output that only a
    ReLU reads, the shortcut branch of a residual sum) is recomputed when a chosen copy reads it, with that copy's
    target and no later control operation, and is left alone when nothing recomputed reads it."""
    spec = SPECS[sname]()
    g0, ids = model.build(spec)
    gam0 = g0.gamma()
    n0 = len(g0.nodes)
    cons_of = dict(select(g0, gam0, Params()))
    # the late-read tensors with the most forward-only tensors behind them (residual sums in the ResNet)
    groups = sorted((forward_only_ancestors(g0, cons_of, u) for u in cons_of), key=len, reverse=True)[:3]
    assert len(groups[0]) >= 2
    lonely = next(n.id for n in g0.nodes if not n.is_var and n.phase == FWD and n.id not in cons_of
                  and not any(n.id in grp for grp in groups) and g0.readers(n.id))
    chosen = sorted({u for grp in groups for u in grp} | {lonely})
    p = Params(recompute_ops=ALL_OPS, recompute_set=chosen, fuse_swapins=True)
    g1 = g0.copy()
    st = rewrite(g1, p)
    gam1 = g1.gamma()
    by_name = {n.name: n for n in g0.nodes}
    copies = [n for n in g1.nodes[n0:] if n.name.endswith("/recompute")]
    copy_of = {by_name[c.name[:-len("/recompute")]].id: c.id for c in copies}
    assert sorted(copy_of) == sorted(set(chosen) - {lonely}) and st.recomputed == len(copies)
    restored = lambda v: g1.inputs(g1.inputs(v)[0])[0] if g1.nodes[v].op == "swap_in" else v
    for u, cid in copy_of.items():
        for a, b in zip(g0.inputs(u), g1.inputs(cid)):
            assert restored(b) == copy_of.get(a, a)
        (ctl,) = g1.control_inputs(cid)
        assert ctl < n0 and gam0[u] < gam0[ctl]
        for v in cons_of.get(u, ()):
            assert cid in [restored(i) for i in g1.inputs(v)] and u not in g1.inputs(v)
            assert gam1[cid] < gam1[v]
        readers = [v for v in g1.readers(cid) if v in copy_of.values()]
        for v in readers:
            (ctl_v,) = g1.control_inputs(v)
            assert ctl <= ctl_v and gam1[cid] < gam1[v]
        if u not in cons_of:
            # serves copies alone; the forward readers of the original still read the original
            assert readers and all(v in copy_of.values() for v in g1.readers(cid))
            assert sorted(g1.readers(u)) == sorted(g0.readers(u))
    assert not [n for n in g1.nodes[n0:] if n.name == g0.nodes[lonely].name + "/recompute"]
    t = W.make_tensors(spec, affine="random")
    a = evaluate.run(g0, t)
    b = evaluate.run(g1, t)
    for name, v in ids.items():
        assert np.array_equal(np.asarray(a[v]), np.asarray(b[v])), name
    for u, cid in copy_of.items():
        assert np.array_equal(np.asarray(a[u]), np.asarray(b[cid]))
