"""Host logic of the library (no GPU): exported symbols, graph building and shape checks, the
topological ordering, the rewriter against the oracle's rewriter on the same graph, the memory
planner against the oracle's lifetime simulation, the budget search and the error paths."""
import os
import re

import pytest

import workloads as W
import paper_1807_02037_amd as L
from paper_1807_02037_amd import abi as A
from oracle import rewrite as orw
from helpers import to_oracle_graph

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SPECS = {
    "chain": lambda: W.tiny_chain(),
    "stage": lambda: W.bottleneck_stage(batch=2, size=8, cin=32, width=8, blocks=3),
    "resnet": lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(2, 2, 1), base=8),
    "unet": lambda: W.unet3d(batch=1, size=8, base=8, levels=3, classes=4, cin=1),
}


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lms.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lms_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 25
    lib = A.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(A.EXPORTS)
    assert b"gfx950" in lib.lms_version()


def test_shapes_and_backward_structure():
    g, ids = L.build_graph(W.tiny_chain())
    info = g.node_info(ids["conv3"])
    assert [info.dims[i] for i in range(info.ndim)] == [2, 32, 32, 16] and info.phase == A.FWD
    gw = g.node_info(ids["grad/conv1.w"])
    assert [gw.dims[i] for i in range(gw.ndim)] == [3, 3, 3, 16] and gw.dtype == A.F32 and gw.phase == A.BWD
    # the input batch is not learnable: no data gradient of the first convolution
    names = [g.node_info(i).name.decode() for i in range(g.node_count())]
    assert "conv1/dgrad" not in names and "conv2/dgrad" in names
    # every parameter has a gradient node
    for n in names:
        if "." in n and not n.startswith("grad/") and "/" not in n:
            assert "grad/" + n in names, n
    g2, ids2 = L.build_graph(W.resnet50(batch=1, size=32, classes=10))
    assert g2.node_info(ids2["fc"]).dims[3] == 10 and g2.node_info(ids2["s5b3c"]).dims[1] == 1
    assert g2.node_info(ids2["grad/stem.scale"]).dims[0] == 64


def test_bad_arguments_are_errors_not_crashes():
    g = L.Graph()
    x = g.add_variable("x", A.BF16, (1, 8, 8, 4), A.VAR_INPUT)
    w = g.add_variable("w", A.BF16, (3, 3, 5, 8), A.VAR_PARAM)       # C mismatch
    with pytest.raises(L.LmsError) as e:
        g.add_op("c", A.OP_CONV, [x, w], stride=1, pad=1)
    assert e.value.status == A.EINVAL and "filter C" in str(e.value)
    with pytest.raises(L.LmsError):
        g.add_op("c", A.OP_CONV, [x], stride=1, pad=1)                 # wrong input count
    with pytest.raises(L.LmsError):
        g.add_op("c", A.OP_CONV, [x, 99], stride=1, pad=1)             # unknown node
    w2 = g.add_variable("w2", A.BF16, (3, 3, 4, 8), A.VAR_PARAM)
    c = g.add_op("c", A.OP_CONV, [x, w2], stride=1, pad=1, flags=A.F_RELU)
    d = g.add_op("d", A.OP_MAXPOOL, [c], filt=(2, 2), stride=2)
    with pytest.raises(L.LmsError) as e:
        g.add_control_edge(d, x)                                       # no control edge into a variable
    assert e.value.status == A.EINVAL
    with pytest.raises(L.LmsError) as e:
        g.add_control_edge(d, c)                                       # would close a cycle
    assert e.value.status == A.ECYCLE
    g.add_control_edge(c, d)
    with pytest.raises(L.LmsError):
        g.build_backward(d)                                            # not a loss
    with pytest.raises(L.LmsError):
        g.rewrite(lb=-1)
    # the pinned-pool helper checks its arguments before it touches the device
    import ctypes as C
    p = C.c_void_p()
    assert A.lib().lms_pinned_alloc(0, C.byref(p)) == A.EINVAL and "lms_pinned_alloc" in A.lib().lms_last_error().decode()
    assert A.lib().lms_pinned_alloc(4096, None) == A.EINVAL
    assert A.lib().lms_pinned_free(None) == A.OK


@pytest.mark.parametrize("name", list(SPECS))
def test_topological_ordering_matches_oracle(name):
    g, ids = L.build_graph(SPECS[name]())
    og, infos = to_oracle_graph(g)
    gam = og.gamma()
    assert g.topo_order() == [gam[i] for i in range(len(infos))]
    assert [info.gamma for info in infos] == [gam[i] for i in range(len(infos))]
    for info in infos:
        assert (info.gamma == 0) == bool(info.is_variable)


def test_control_edge_raises_order_like_fig2c():
    # Section 3.2, Figure 2(c): a control edge pushes the target one order later
    g = L.Graph()
    x = g.add_variable("x", A.BF16, (1, 4, 4, 8), A.VAR_INPUT)
    h = g.add_op("h", A.OP_MAXPOOL, [x], filt=(1, 1), stride=1)
    f = g.add_op("f", A.OP_MAXPOOL, [h], filt=(1, 1), stride=1)
    f1 = g.add_op("f1", A.OP_CONCAT, [f, x])
    f2 = g.add_op("f2", A.OP_MAXPOOL, [f], filt=(1, 1), stride=1)
    g.add_update_edge(f2, x)
    assert g.topo_order() == [0, 1, 2, 3, 3]
    g.add_control_edge(f2, f1)
    assert g.topo_order() == [0, 1, 2, 4, 3]


PARAMS = [
    dict(), dict(lb=2), dict(lb=3, ub=5), dict(ctrld_strategy=A.DIRECT_ORDER), dict(ctrld_strategy=A.DIRECT_ORDER, lb=4),
    dict(fuse_swapins=1), dict(n_tensors=3), dict(n_tensors=0), dict(swap_branches=1, branch_threshold=3),
    dict(swap_branches=1, fuse_swapins=1, lb=2), dict(fuse_swapins=1, fuse_distance=2),
    dict(excl_type=A.OP_CONV), dict(incl_type=A.OP_CONV, excl_scope="conv2"), dict(incl_scope="b2"),
    dict(starting_op_name="conv2"),
    # Table 2's list-valued fields with more than one entry
    dict(excl_types=[A.OP_CONV, A.OP_MAXPOOL]), dict(incl_types=[A.OP_CONV, A.OP_CONCAT], excl_scopes=["conv2", "b1", "e0"]),
    dict(incl_scopes=["b2", "b3", "conv3", "s3", "d"]), dict(starting_op_names=["conv2", "b2a", "s3b1a", "e1a"], fuse_swapins=1),
]


def oracle_params(kw):
    p = orw.Params()
    for k, v in kw.items():
        if k == "ctrld_strategy":
            p.ctrld_strategy = {A.CHAIN_RULE: "chain_rule", A.DIRECT_ORDER: "direct_order"}[v]
        elif k in ("fuse_swapins", "swap_branches"):
            setattr(p, k, bool(v))
        elif k == "fuse_distance":
            p.fuse_distance = v if v >= 0 else orw.INF
        elif k in ("excl_type", "excl_types", "incl_type", "incl_types"):
            setattr(p, k if k.endswith("s") else k + "s", [f"op{o}" for o in ([v] if isinstance(v, int) else v)])
        elif k in ("excl_scope", "excl_scopes", "incl_scope", "incl_scopes", "starting_op_name", "starting_op_names"):
            setattr(p, k if k.endswith("s") else k + "s", [v] if isinstance(v, str) else list(v))
        else:
            setattr(p, k, v)
    return p


def rewritten_signature(og):
    """What a rewrite decided, independent of vertex numbering of the inserted operations:
    {(producer, frozenset(consumers of one swap-in)): (control op, swap-out label, swap-in label)}."""
    sig = {}
    for n in og.nodes:
        if n.op != "swap_in":
            continue
        so = og.inputs(n.id)[0]
        u = og.inputs(so)[0]
        ctl = og.control_inputs(n.id)
        sig[(u, frozenset(og.readers(n.id)))] = (tuple(ctl), og.nodes[so].label, n.label)
    return sig


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_rewriter_matches_oracle_rewriter(name, pi):
    kw = PARAMS[pi]
    g, ids = L.build_graph(SPECS[name]())
    og0, _ = to_oracle_graph(g)
    ost = orw.rewrite(og0_copy := og0.copy(), oracle_params(kw))
    st = g.rewrite(**kw)
    og1, infos = to_oracle_graph(g)
    assert (st.tensors_swapped, st.swap_outs, st.swap_ins, st.control_edges) == \
           (ost.tensors, ost.swap_outs, ost.swap_ins, ost.control_edges)
    # same tensors, same consumer groups, same control operations and the labels of Figure 3
    assert rewritten_signature(og1) == rewritten_signature(og0_copy)
    # and the structural invariants hold for the library's graph in its own right
    assert orw.contract_swaps(og1) == orw.contract_swaps(og0)
    og1.gamma()                                            # acyclic
    gam0 = og0.gamma()
    for n in og1.nodes:
        if n.op == "swap_in":
            (ctl,) = og1.control_inputs(n.id)
            u = og1.inputs(og1.inputs(n.id)[0])[0]
            for v in og1.readers(n.id):
                assert gam0[u] < gam0[ctl] < gam0[v]
        if n.op in ("swap_in", "swap_out"):
            assert n.placement == "host" and infos[n.id].phase == A.SWAP
    # vertices that existed before keep their order
    for i, info in enumerate(infos):
        if info.op not in (A.OP_SWAP_OUT, A.OP_SWAP_IN):
            assert info.gamma == gam0[i]


@pytest.mark.parametrize("name", list(SPECS))
def test_own_placement_is_valid(name):
    g, ids = L.build_graph(SPECS[name]())
    og0, _ = to_oracle_graph(g)
    need = g.memory_need()[1]
    floor = g.clone().rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    budget = (need + floor) // 2
    st = g.rewrite(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN)
    assert 0 < st.tensors_swapped and st.arena_needed_after <= budget
    og1, _ = to_oracle_graph(g)
    assert orw.contract_swaps(og1) == orw.contract_swaps(og0)
    gam0 = og0.gamma()
    og1.gamma()
    for n in og1.nodes:
        if n.op == "swap_in":
            (ctl,) = og1.control_inputs(n.id)
            u = og1.inputs(og1.inputs(n.id)[0])[0]
            for v in og1.readers(n.id):
                assert gam0[u] < gam0[ctl] < gam0[v]


def with_fetch(og, order, nbytes):
    """The library keeps tensors nobody reads (the loss, parameter gradients) until the step ends,
    as if a final fetch operation consumed them; give the oracle's graph that operation."""
    unread = [n.id for n in og.nodes if not n.is_var and not og.readers(n.id) and n.op != "swap_out"]
    f = og.add_op("fetch", "fetch", unread, "upd")
    nbytes[f] = 0
    return list(order) + [f]


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("kw", [None, dict(), dict(fuse_swapins=1, lb=2)])
def test_peak_live_bytes_matches_lifetime_simulation(name, kw):
    """The planner's peak of live bytes equals the oracle's reference-count simulation (Section 3.5)
    on the same execution order, once in-place accumulation and workspaces are accounted for."""
    g, ids = L.build_graph(SPECS[name]())
    if kw is not None:
        g.rewrite(**kw)
    og, infos = to_oracle_graph(g)
    order = g.schedule()
    assert sorted(order) == list(range(len(infos)))
    pos = {v: i for i, v in enumerate(order)}
    for e in og.edges:                                     # the order respects every read and control edge
        if e.action != "update" and not og.nodes[e.dst].is_var:
            assert pos[e.src] < pos[e.dst]
    rnd = lambda b: (b + 255) // 256 * 256
    nbytes = {i: rnd(infos[i].bytes) for i in range(len(infos))}
    order = with_fetch(og, order, nbytes)
    plain, trace = orw.peak_live_bytes(og, order, nbytes)
    ws_peak = max(trace[pos[i]] + rnd(infos[i].workspace_bytes) for i in range(len(infos)))
    peak_live, arena = g.memory_need()
    assert arena >= peak_live
    # in-place accumulation can only lower the need; never below the largest single tensor + workspace
    assert peak_live <= max(plain, ws_peak)
    assert peak_live >= max(nbytes[i] for i in range(len(infos)) if not infos[i].is_variable)
    if not any(info.flags & (A.F_ADDEND) or info.op in (A.OP_GRAD_SUM, A.OP_MSE_GRAD) for info in infos):
        assert peak_live == max(plain, ws_peak)


def test_forward_only_peak_equals_simulation_exactly():
    # without backward there is no in-place accumulation: the two numbers must agree exactly
    g, ids = L.build_graph(W.bottleneck_stage(batch=2, size=8, cin=32, width=8), backward=False)
    og, infos = to_oracle_graph(g)
    order = g.schedule()
    rnd = lambda b: (b + 255) // 256 * 256
    pos = {v: i for i, v in enumerate(order)}
    nbytes = {i: rnd(infos[i].bytes) for i in range(len(infos))}
    order = with_fetch(og, order, nbytes)
    plain, trace = orw.peak_live_bytes(og, order, nbytes)
    ws_peak = max(trace[pos[i]] + rnd(infos[i].workspace_bytes) for i in range(len(infos)))
    assert g.memory_need()[0] == max(plain, ws_peak)


def needs_by_n(spec, **kw):
    out = []
    n = 0
    while True:
        g, _ = L.build_graph(spec)
        st = g.rewrite(n_tensors=n, **kw)
        out.append(g.memory_need()[1])
        if st.tensors_swapped < n:
            return out[:-1]
        n += 1


def test_budget_search_swaps_exactly_two_on_the_tiny_chain():
    """Config 1: a budget B with need(2 tensors) <= B < need(1 tensor) makes the planner swap exactly 2."""
    spec = W.tiny_chain()
    need = needs_by_n(spec, fuse_swapins=1)
    assert len(need) >= 4 and need[2] < need[1] <= need[0]
    g, ids = L.build_graph(spec)
    st = g.rewrite(budget_bytes=need[2], fuse_swapins=1)
    assert st.tensors_swapped == 2 and st.swap_outs == 2 and st.swap_ins == 2
    assert st.arena_needed_after <= need[2] < st.arena_needed_before
    swapped = sorted(g.node_info(i).name.decode() for i in range(g.node_count()) if g.node_info(i).op == A.OP_SWAP_OUT)
    assert swapped == ["conv1/swap_out", "conv2/swap_out"]     # breadth-first from the input
    # a budget that needs no swapping leaves the graph alone
    g2, _ = L.build_graph(spec)
    assert g2.rewrite(budget_bytes=need[0]).tensors_swapped == 0


def test_infeasible_budget_is_reported():
    spec = W.bottleneck_stage(batch=2, size=8, cin=32, width=8)
    g, _ = L.build_graph(spec)
    n0 = g.node_count()
    with pytest.raises(L.LmsError) as e:
        g.rewrite(budget_bytes=4096, fuse_swapins=1)
    assert e.value.status == A.EBUDGET and "below" in str(e.value)
    assert g.node_count() == n0                                  # graph left unchanged
    with pytest.raises(L.LmsError) as e:
        g.rewrite()
        g.rewrite()                                              # rewriting twice is refused
    assert e.value.status == A.EINVAL


def test_config2_half_footprint_budget_is_feasible():
    g, _ = L.build_graph(W.bottleneck_stage())
    peak, arena = g.memory_need()
    st = g.rewrite(budget_bytes=arena // 2, fuse_swapins=1, ctrld_strategy=A.OWN)
    assert st.arena_needed_after <= arena // 2 and st.tensors_swapped >= 4
    assert st.swapped_bytes_out == st.swapped_bytes_in > 2e8


def test_own_selection_drops_tensors_the_budget_does_not_need():
    """The library's own strategy removes, largest first, swapped tensors without which the plan still fits: never
    more tensors or bytes than the breadth-first prefix of the paper's procedure, and the plan still fits the budget."""
    spec = W.unet3d(batch=1, size=128)                      # planning only: no tensors are allocated
    g0, _ = L.build_graph(spec)
    need = g0.memory_need()[1]
    fewer = False
    for frac in (0.5, 0.6, 0.7):
        budget = int(need * frac)
        gp, go = g0.clone(), g0.clone()
        sp = gp.rewrite(budget_bytes=budget, fuse_swapins=1)
        so = go.rewrite(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN)
        assert so.arena_needed_after <= budget and sp.arena_needed_after <= budget
        assert so.tensors_swapped <= sp.tensors_swapped and so.swapped_bytes_out <= sp.swapped_bytes_out
        fewer = fewer or so.swapped_bytes_out < sp.swapped_bytes_out
    assert fewer


def test_bias_gradient_node_is_served_by_the_weight_gradient_node_when_bound_to_caller_memory():
    """A COLSUM node (per-channel sum of dy: the shift gradient) whose output is declared external plans no workspace
    of its own, the CONV_WGRAD node of the same dy reserves the partial sums instead; without the declaration both keep
    their own (the executor then runs the separate pass).  Swapping dy's consumers elsewhere does not change the pairing."""
    import workloads as W
    from paper_1807_02037_amd.models import build_graph
    spec = W.resnet50(batch=4, size=32)
    g = build_graph(spec)[0]
    infos = [g.node_info(i) for i in range(g.node_count())]
    col = [i for i in infos if i.op == A.OP_COLSUM and not i.is_variable]
    assert len(col) >= 53
    paired = 0
    for c in col:
        dz = g.node_inputs(c.id)[0]
        host = [w for w in infos[max(0, c.id - 8):c.id] if w.op == A.OP_CONV_WGRAD and g.node_inputs(w.id)[1] == dz]
        if infos[dz].dtype != A.BF16 or not host:
            continue
        paired += 1
        assert c.workspace_bytes == 0
        w = host[-1]
        ws_paired = w.workspace_bytes
        g.set_external(c.id, False)
        assert g.node_info(c.id).workspace_bytes > 0
        assert g.node_info(w.id).workspace_bytes <= ws_paired
        g.set_external(c.id, True)
        assert g.node_info(w.id).workspace_bytes == ws_paired
    assert paired >= 52
    before = {c.id: g.node_info(c.id).workspace_bytes for c in col}
    g.rewrite(n_tensors=-1, fuse_swapins=1)
    assert before == {c.id: g.node_info(c.id).workspace_bytes for c in col}


@pytest.mark.parametrize("batch,budget_gb", [(1276, 16), (3796, 16)])
def test_fused_bias_gradient_is_scheduled_after_the_weight_gradient_that_writes_it(batch, budget_gb):
    """In a rewritten graph a weight-gradient node may have to wait for a swap-in or a recomputed copy of its input
    while the column sum of the same dy could run at once.  The column sum comes out of the weight-gradient pass, so
    the schedule must keep it (and with it the update operation that reads it) behind that node."""
    import workloads as W
    from paper_1807_02037_amd.models import build_graph
    g = build_graph(W.resnet50(batch=batch, size=224), lr=1e-4)[0]
    st = g.rewrite(budget_bytes=budget_gb * 10**9, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=2, encoded_swaps=1)
    assert st.recomputed > 0
    infos = [g.node_info(i) for i in range(g.node_count())]
    pos = {v: i for i, v in enumerate(g.schedule())}
    by_name = {i.name.decode(): i.id for i in infos}
    origin = lambda v: origin(g.node_inputs(v)[0]) if infos[v].op in (A.OP_SWAP_IN, A.OP_SWAP_OUT) else v
    checked = delayed = 0
    for c in infos:
        if c.op != A.OP_COLSUM or c.is_variable:
            continue
        dz = origin(g.node_inputs(c.id)[0])
        hosts = [w for w in infos[max(0, c.id - 8):c.id] if w.op == A.OP_CONV_WGRAD and origin(g.node_inputs(w.id)[1]) == dz]
        if infos[dz].dtype != A.BF16 or not hosts:
            continue
        w = hosts[-1]
        assert pos[w.id] < pos[c.id], (c.name, w.name)
        upd = by_name["update/" + c.name.decode()[len("grad/"):]]
        assert pos[c.id] < pos[upd]
        checked += 1
        # the case the rule is for: the node's first input is not there when dy is (it is swapped in or computed again)
        delayed += pos[g.node_inputs(w.id)[0]] > pos[dz]
    assert checked >= 52 and delayed > 0
    # Section 3.2: the operation that updates a variable runs after every other reader of that variable (they were all
    # created before it, the recomputed copies as repetitions of forward operations): none may see the new value
    readers = {}
    for i in infos:
        if not i.is_variable:
            for u in g.node_inputs(i.id):
                if infos[u].is_variable:
                    readers.setdefault(u, []).append(i.id)
    updates = [i for i in infos if i.name.startswith(b"update/")]
    assert len(updates) == 161
    late_readers = 0
    for u in updates:
        var = by_name[u.name.decode()[len("update/"):]]
        for r in readers[var]:
            if r != u.id:
                assert pos[r] < pos[u.id], (u.name, infos[r].name)
                late_readers += r > u.id                    # a copy inserted by the rewriter
    assert late_readers > 0
