"""The library's chained recomputation pass and its hybrid planner (host logic, no GPU): the pass against the
oracle's pass on the same graph and parameters, and the planner's choice under a budget (valid, fits, never worse
than swaps alone in its own estimate, fewer bytes over the link)."""
import pytest

import workloads as W
import paper_1807_02037_amd as L
from paper_1807_02037_amd import abi as A
from oracle import rewrite as orw
from helpers import to_oracle_graph
from test_lib_host import oracle_params, rewritten_signature

SPECS = {
    "chain": lambda: W.tiny_chain(),
    "pool_net": lambda: W.pool_net(),
    "updown_net": lambda: W.updown_net(),
    "stage": lambda: W.bottleneck_stage(batch=2, size=8, cin=32, width=8, blocks=3),
    "resnet": lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(2, 2, 1), base=8),
    "unet": lambda: W.unet3d(batch=1, size=8, base=8, levels=3, classes=4, cin=1),
}
RECOMPUTABLE = tuple(f"op{c}" for c in (A.OP_CONV, A.OP_TCONV, A.OP_MAXPOOL, A.OP_CONCAT, A.OP_GAP))
PARAMS = [dict(recompute_depth=1), dict(recompute_depth=2, fuse_swapins=1), dict(recompute_depth=3, fuse_swapins=1, lb=2),
          dict(recompute_depth=2, ctrld_strategy=A.DIRECT_ORDER, n_tensors=0), dict(recompute_depth=40, n_tensors=2, fuse_swapins=1),
          dict(recompute_depth=2, swap_branches=1, branch_threshold=2, fuse_swapins=1), dict(recompute_depth=4, lb=3, ub=8)]


def is_copy(n):
    return "/recompute" in n.name and n.op not in ("swap_in", "swap_out")


def copies_signature(og, n0):
    """{recomputed producer name: (op, inputs with copies named by the tensor they repeat, control op, label, phase,
    readers that are not copies)}; an input the swap pass rerouted through a swap-in is named by what it restores."""
    names = {n.id: n.name.split("/recompute")[0] + "'" for n in og.nodes[n0:] if is_copy(n)}

    def origin(v):
        while og.nodes[v].op in ("swap_in", "swap_out"):
            v = og.inputs(v)[0]
        return names.get(v, v)
    sig = {}
    for n in og.nodes[n0:]:
        if n.id in names:
            sig[names[n.id]] = (n.op, tuple(origin(i) for i in og.inputs(n.id)), tuple(og.control_inputs(n.id)), n.label, n.phase,
                                frozenset(v for v in og.readers(n.id) if v < n0))
    return sig


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_chained_pass_matches_oracle(name, pi):
    kw = dict(PARAMS[pi], recompute=2)
    g, ids = L.build_graph(SPECS[name]())
    n0 = g.node_count()
    og0, _ = to_oracle_graph(g)
    op = oracle_params({k: v for k, v in kw.items() if k not in ("recompute",)})
    op.recompute_ops = RECOMPUTABLE
    og_ref = og0.copy()
    ost = orw.rewrite(og_ref, op)
    st = g.rewrite(**kw)
    og1, infos = to_oracle_graph(g)
    assert st.recomputed == ost.recomputed > 0
    assert (st.tensors_swapped, st.swap_outs, st.swap_ins, st.control_edges, st.unrewritten) == \
           (ost.tensors, ost.swap_outs, ost.swap_ins, ost.control_edges, ost.unrewritten)
    assert copies_signature(og1, n0) == copies_signature(og_ref, n0)
    assert g.node_count() == len(og_ref.nodes)
    og1.gamma()                                            # acyclic
    # the swap decisions (tensor, consumers, control op, labels) agree too; consumers that are copies are matched by
    # the tensor they repeat, since the two sides number inserted vertices differently
    def swaps(og):
        names = {n.id: n.name.split("/recompute")[0] + "'" for n in og.nodes[n0:] if is_copy(n)}
        return {(u, frozenset(names.get(v, v) for v in cons)): val for (u, cons), val in rewritten_signature(og).items()}
    assert swaps(og1) == swaps(og_ref)
    # the library's execution order runs every copy after the copies it reads and before its consumers
    order = g.schedule()
    pos = {v: i for i, v in enumerate(order)}
    for n in og1.nodes[n0:]:
        if is_copy(n):
            for i in og1.inputs(n.id):
                assert pos[i] < pos[n.id]
            for v in og1.readers(n.id):
                assert pos[n.id] < pos[v]


@pytest.mark.parametrize("name", ["stage", "resnet", "unet", "pool_net"])
def test_hybrid_planner_fits_and_moves_fewer_bytes(name):
    spec = SPECS[name]()
    g_sw, _ = L.build_graph(spec)
    need = g_sw.memory_need()[1]
    floor = g_sw.clone().rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    budget = (need + 3 * floor) // 4
    s_sw = g_sw.rewrite(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN)
    g_hy, _ = L.build_graph(spec)
    og0, _ = to_oracle_graph(g_hy)
    n0 = g_hy.node_count()
    s_hy = g_hy.rewrite(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2)
    assert s_hy.arena_needed_after <= budget and s_sw.arena_needed_after <= budget
    assert s_hy.swapped_bytes_out <= s_sw.swapped_bytes_out
    assert s_hy.recomputed > 0 and s_hy.swapped_bytes_out < s_sw.swapped_bytes_out
    # judged by the planner's own played-through step, the chosen plan is no slower than the plan with swaps alone
    assert 0 < s_hy.estimated_ms <= s_sw.estimated_ms
    assert_contracts_to(g_hy, og0, n0)


def assert_contracts_to(g, og0, n0):
    """Contracting the swaps and redirecting the readers of every copy to its original gives back the original read
    edges; a copy reads what its original reads (through copies and swaps)."""
    og1, _ = to_oracle_graph(g)
    og1.gamma()
    back = {}
    for n in og1.nodes[n0:]:
        if is_copy(n):
            back[n.id] = next(m.id for m in og1.nodes[:n0] if m.name == n.name.split("/recompute")[0])
    def origin(v):
        while og1.nodes[v].op in ("swap_in", "swap_out"):
            v = og1.inputs(v)[0]
        return back.get(v, v)
    edges = sorted((origin(e.src), e.dst, e.slot) for e in og1.edges
                   if e.action == "read" and e.dst < n0)
    ref = sorted((e.src, e.dst, e.slot) for e in og0.edges if e.action == "read")
    assert edges == ref
    for cid, u in back.items():
        assert [origin(i) for i in og1.inputs(cid)] == list(og0.inputs(u))
    return og1, back


def test_hybrid_planner_recomputes_a_shortcut_branch_for_the_copy_that_reads_it():
    """ResNet-50 at 224x224, 1.5 times the batch that fits 16 GB: the residual sum of the first block is recomputed,
    and with it the projection shortcut that nothing in the backward phase reads: no tensor crosses the link."""
    g, _ = L.build_graph(W.resnet50(batch=1278, size=224))
    og0, _ = to_oracle_graph(g)
    n0 = g.node_count()
    st = g.rewrite(budget_bytes=16 * 10**9, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2, encoded_swaps=1)
    assert st.arena_needed_after <= 16 * 10**9 < st.arena_needed_before
    og1, back = assert_contracts_to(g, og0, n0)
    by_name = {og0.nodes[u].name: c for c, u in back.items()}
    assert "s2b1p" in by_name and "s2b1c" in by_name
    assert og1.readers(by_name["s2b1p"]) == [by_name["s2b1c"]]            # the copy of the sum alone reads it
    assert sorted(og1.readers(back[by_name["s2b1p"]])) == sorted(og0.readers(back[by_name["s2b1p"]]))
    assert st.tensors_swapped == 0 and st.recomputed == len(back)
    # against the same budget with swaps alone the estimate says why
    g_sw, _ = L.build_graph(W.resnet50(batch=1278, size=224))
    s_sw = g_sw.rewrite(budget_bytes=16 * 10**9, fuse_swapins=1, ctrld_strategy=A.OWN, encoded_swaps=1)
    assert s_sw.tensors_swapped > 0 and st.estimated_ms < s_sw.estimated_ms


def test_budget_below_the_swap_floor_is_still_an_error_with_the_planner():
    g, _ = L.build_graph(SPECS["stage"]())
    floor = g.clone().rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    floors = [floor]
    for d in (1, 2, 3):
        floors.append(g.clone().rewrite(fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2, recompute_depth=d).arena_needed_after)
    with pytest.raises(L.LmsError) as e:
        g.rewrite(budget_bytes=min(floors) // 2, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2)
    assert e.value.status == A.EBUDGET


def test_estimated_step_follows_the_machine_figures():
    """lms_rewrite_stats.estimated_ms of a fixed plan (swaps alone: the plan does not depend on the estimate): never
    below the unswapped step, shorter with a faster link, with the encoded transfer and with a faster device."""
    spec = SPECS["resnet"]()
    need = L.build_graph(spec)[0].memory_need()[1]
    floor = L.build_graph(spec)[0].rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    budget = (need + floor) // 2

    def est(**kw):
        g, _ = L.build_graph(spec)
        st = g.rewrite(budget_bytes=kw.pop("budget", budget), fuse_swapins=1, ctrld_strategy=A.OWN, **kw)
        return st.estimated_ms, st
    plain, st = est()
    assert st.tensors_swapped > 0 and plain > 0
    unswapped, st0 = est(budget=2 * need)
    assert st0.tensors_swapped == 0 and 0 < unswapped <= plain
    slow, fast = est(link_gbs=5.0)[0], est(link_gbs=500.0)[0]
    assert slow > plain >= fast >= unswapped
    assert est(encoded_swaps=1)[0] <= plain
    assert est(device_tflops=5.0, hbm_gbs=50.0)[0] > plain > est(device_tflops=5000.0, hbm_gbs=50000.0)[0]
    # without a budget nothing is estimated
    g, _ = L.build_graph(spec)
    assert g.rewrite(fuse_swapins=1).estimated_ms == 0
