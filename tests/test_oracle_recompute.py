"""Pins of the oracle's recomputation pass: structure of the inserted copies, unchanged values, and the memory
effect (a recomputed tensor no longer lives from the forward into the backward phase)."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate, model
from oracle.graph import READ, CONTROL, FWD, BWD
from oracle.rewrite import Params, rewrite, peak_live_bytes

SPECS = {
    "pool_net": lambda: W.pool_net(),
    "updown_net": lambda: W.updown_net(),
    "unet": lambda: W.unet3d(batch=1, size=8, base=4, levels=3, classes=3),
    "resnet": lambda: W.resnet50(batch=1, size=16, classes=4, stage_blocks=(1, 1), base=4),
}
CHEAP = ("maxpool", "concat", "gap")
PARAMS = [Params(recompute=True), Params(recompute=True, fuse_swapins=True, lb=2),
          Params(recompute=True, ctrld_strategy="direct_order", n_tensors=0),
          Params(recompute=True, swap_branches=True, branch_threshold=2, fuse_swapins=True)]


@pytest.mark.parametrize("sname", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_copies_are_valid_and_change_no_value(sname, pi):
    spec = SPECS[sname]()
    p = PARAMS[pi]
    g0, ids = model.build(spec)
    g1 = g0.copy()
    st = rewrite(g1, p)
    gam0 = g0.gamma()
    g1.gamma()                                                     # acyclic
    n0 = len(g0.nodes)
    copies = [n for n in g1.nodes[n0:] if n.op in CHEAP]
    assert len(copies) == st.recomputed
    by_name = {n.name: n for n in g0.nodes}
    for c in copies:
        src = by_name[c.name.split("/recompute")[0]]
        assert c.op == src.op and c.attrs == src.attrs and src.phase == FWD
        # same inputs in the same slots, unless the swap pass that follows has put a swap-in in between
        ins0 = g0.inputs(src.id)
        ins1 = g1.inputs(c.id)
        assert len(ins0) == len(ins1)
        for a, b in zip(ins0, ins1):
            nb = g1.nodes[b]
            assert b == a or (nb.op == "swap_in" and g1.inputs(g1.inputs(b)[0])[0] == a)
        (ctl,) = g1.control_inputs(c.id)
        assert c.label == gam0[ctl] + 1
        readers = g1.readers(c.id)
        assert readers
        for v in readers:                                          # the trigger lies strictly between producer and consumer
            assert gam0[src.id] < gam0[ctl] < gam0[v]
            assert c.phase == g0.nodes[min(readers, key=lambda r: (gam0[r], r))].phase
    # a cheap tensor that was recomputed has lost the late readers that made it a candidate
    late = Params(**{**p.__dict__, "n_tensors": -1, "recompute": False})
    from oracle.rewrite import select
    for u, cons in select(g0, gam0, late):
        if g0.nodes[u].op in CHEAP:
            left = [v for v in g1.readers(u) if v in cons]
            assert len(left) <= st.unrewritten
    # values: every original vertex evaluates to the same bits
    t = W.make_tensors(spec, affine="random")
    a = evaluate.run(g0, t)
    b = evaluate.run(g1, t)
    for name, v in ids.items():
        assert np.array_equal(np.asarray(a[v]), np.asarray(b[v])), name


def test_cheap_tensors_are_recomputed_not_swapped():
    spec = SPECS["unet"]()
    g0, ids = model.build(spec)
    g_swap, g_rec = g0.copy(), g0.copy()
    s_swap = rewrite(g_swap, Params(fuse_swapins=True))
    s_rec = rewrite(g_rec, Params(fuse_swapins=True, recompute=True))
    cheap_swapped = [u for u in s_swap.swapped if g0.nodes[u].op in CHEAP]
    assert cheap_swapped                                            # pools and concatenations do cross into the backward phase
    assert not [u for u in s_rec.swapped if g0.nodes[u].op in CHEAP]
    assert s_rec.recomputed >= len(cheap_swapped)
    # the other tensors are swapped as before; an input of a copy that had no late reader before has one now
    kept = [u for u in s_swap.swapped if g0.nodes[u].op not in CHEAP]
    assert set(kept) <= set(s_rec.swapped)
    copy_inputs = {a for u in cheap_swapped for a in g0.inputs(u)}
    assert set(s_rec.swapped) - set(kept) <= copy_inputs
    # with nothing swapped at all, recomputation alone lowers the peak of live bytes
    g_only = g0.copy()
    rewrite(g_only, Params(recompute=True, n_tensors=0))
    t = W.make_tensors(spec)
    vals = evaluate.run(g0, t)
    vals1 = evaluate.run(g_only, t)
    nbytes0 = {v: 2 * int(np.asarray(vals[v]).size) for v in range(len(g0.nodes)) if not g0.nodes[v].is_var}
    nbytes1 = {v: 2 * int(np.asarray(vals1[v]).size) for v in range(len(g_only.nodes)) if not g_only.nodes[v].is_var}
    order0 = [n.id for n in g0.nodes if not n.is_var]
    gam1 = g_only.gamma()
    order1 = sorted((n.id for n in g_only.nodes if not n.is_var), key=lambda v: (gam1[v], v))
    assert peak_live_bytes(g_only, order1, nbytes1) < peak_live_bytes(g0, order0, nbytes0)
