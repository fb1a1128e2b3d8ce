"""The library's recomputation pass (host logic, no GPU) against the oracle's rewriter run with the same parameters."""
import pytest

import workloads as W
import paper_1807_02037_amd as L
from paper_1807_02037_amd import abi as A
from oracle import rewrite as orw
from helpers import to_oracle_graph
from test_lib_host import oracle_params, rewritten_signature

SPECS = {
    "pool_net": lambda: W.pool_net(),
    "updown_net": lambda: W.updown_net(),
    "resnet": lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(2, 2, 1), base=8),
    "unet": lambda: W.unet3d(batch=1, size=8, base=8, levels=3, classes=4, cin=1),
}
CHEAP = tuple(f"op{c}" for c in (A.OP_MAXPOOL, A.OP_CONCAT, A.OP_GAP))
PARAMS = [dict(), dict(fuse_swapins=1, lb=2), dict(ctrld_strategy=A.DIRECT_ORDER, n_tensors=0), dict(n_tensors=2),
          dict(swap_branches=1, branch_threshold=2, fuse_swapins=1), dict(fuse_swapins=1, fuse_distance=3, lb=3, ub=8)]


def copies_signature(og, n0):
    """{(cheap producer, consumers of one copy): (op, inputs, control op, label, phase)} of the recomputed copies;
    an input that the swap pass has rerouted through a swap-in is named by the tensor it restores."""
    def origin(v):
        while og.nodes[v].op in ("swap_in", "swap_out"):
            v = og.inputs(v)[0]
        return v
    sig = {}
    for n in og.nodes[n0:]:
        if n.op in CHEAP:
            src = n.name.split("/recompute")[0]
            sig[(src, frozenset(og.readers(n.id)))] = (n.op, tuple(origin(i) for i in og.inputs(n.id)),
                                                       tuple(og.control_inputs(n.id)), n.label, n.phase)
    return sig


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_recompute_pass_matches_oracle(name, pi):
    kw = dict(PARAMS[pi], recompute=1)
    g, ids = L.build_graph(SPECS[name]())
    n0 = g.node_count()
    og0, _ = to_oracle_graph(g)
    op = oracle_params({k: v for k, v in kw.items() if k != "recompute"})
    op.recompute, op.cheap_ops = True, CHEAP
    og_ref = og0.copy()
    ost = orw.rewrite(og_ref, op)
    st = g.rewrite(**kw)
    og1, infos = to_oracle_graph(g)
    assert st.recomputed == ost.recomputed
    if name != "updown_net":
        assert st.recomputed > 0
    assert (st.tensors_swapped, st.swap_outs, st.swap_ins, st.control_edges, st.unrewritten) == \
           (ost.tensors, ost.swap_outs, ost.swap_ins, ost.control_edges, ost.unrewritten)
    assert copies_signature(og1, n0) == copies_signature(og_ref, n0)
    assert rewritten_signature(og1) == rewritten_signature(og_ref)
    assert g.node_count() == len(og_ref.nodes)
    og1.gamma()                                            # acyclic
    # vertices that existed before the swap pass keep the order they have in the graph with the copies
    mid = og0.copy()
    orw.recompute_cheap(mid, op, orw.Stats())
    gam_mid = mid.gamma()
    for i, info in enumerate(infos):
        if i < n0:
            assert info.gamma == gam_mid[i]


def test_recompute_moves_fewer_bytes_at_a_similar_memory_floor():
    spec = W.unet3d(batch=1, size=16, base=8, levels=3, classes=4, cin=1)
    g0, _ = L.build_graph(spec)
    g1, _ = L.build_graph(spec)
    s0 = g0.rewrite(fuse_swapins=1, lb=2)
    s1 = g1.rewrite(fuse_swapins=1, lb=2, recompute=1)
    assert s1.recomputed > 0
    assert s1.swapped_bytes_out < s0.swapped_bytes_out
    # a copy needs its inputs back on the device together, so the floor is not lower than with swaps alone, only close
    assert s0.arena_needed_after < s0.arena_needed_before and s1.arena_needed_after < s1.arena_needed_before
    assert s1.arena_needed_after <= 1.2 * s0.arena_needed_after


def test_rewriting_twice_is_refused_after_recompute():
    g, _ = L.build_graph(W.pool_net())
    g.rewrite(recompute=1, n_tensors=0)
    with pytest.raises(L.LmsError):
        g.rewrite()
