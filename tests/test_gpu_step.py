"""Whole training steps on the GPU against the oracle, and swapped against unswapped runs.

Bars.  The parity gate is the fp64 oracle with every tensor that the GPU path stores in bf16
rounded to bf16 at the same point ("quantisation-matched"): ReLU masks and max-pool winners are
binary decisions taken on stored values, so both sides must take them in the same precision.
Against it, loss, every parameter gradient and every layer output must agree within 1e-2 (max
abs error over max abs value of the tensor), the bound the workload states for bf16.
Against the oracle without any intermediate rounding the loss and the layer outputs must also be
within 1e-2; parameter gradients are held there to 1e-2 plus what bf16 storage of the activations alone moves
them by in the oracle (and to 6e-2 outright on the config 1 and config 2 nets): rounding one forward activation to bf16
(at most 2^-8 of an element) flips ReLU masks downstream and alone moves a weight gradient of the 4-layer
chain by 1.1e-2 (tests/test_oracle_quant.py shows it with the oracle alone), and of the small deep nets used
here (a few positions per channel in the last stages) by tens of percent, even when every later operation is exact.
The gate is also run with every backward gradient rounded where it is produced (no knowledge of which sums and
masks the library fuses): the placement of the backward roundings must not matter.
A rewritten (swapping) run must be bit-identical to the run of the original graph, also with
released blocks poisoned."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate

pytestmark = pytest.mark.gpu

TOL = 1e-2


def rel_err(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


SPECS = {
    "cfg1_tiny_chain": lambda: W.tiny_chain(),
    "cfg2_stage_small": lambda: W.bottleneck_stage(batch=2, size=14, cin=64, width=16, blocks=3),
    "cfg3_resnet_small": lambda: W.resnet50(batch=2, size=64, classes=1000),
    "cfg4_unet_small": lambda: W.unet3d(batch=1, size=16, base=32, levels=4, classes=4, cin=1),
    "pool_net": lambda: W.pool_net(),
    # overlapping pooling over several 16 x 16 tiles with an odd edge, 72 channels (two groups of 64, the second partial)
    "pool_net_ragged": lambda: W.pool_net(batch=2, size=37, cin=8, width=72),
    "updown_net": lambda: W.updown_net(),
    # 2-D transposed convolution wide enough for the pointwise kernels (forward and weight gradient), 11 x 11 inner grid
    "updown_net_2d_wide": lambda: W.updown_net(batch=2, size=22, cin=8, width=48, ndim=2),
}


DEEP = ("cfg3_resnet_small", "cfg4_unet_small")


def run(spec, tensors, rewrite=None, flags=0, steps=1):
    from paper_1807_02037_amd.session import Session
    s = Session(spec, tensors, rewrite=rewrite, flags=flags)
    for _ in range(steps):
        loss, st = s.step()
    return s, loss, st


@pytest.mark.parametrize("name", list(SPECS))
def test_step_matches_oracle(name):
    import paper_1807_02037_amd as L
    spec = SPECS[name]()
    tensors = W.make_tensors(spec, affine="random")
    exact = evaluate.train_step(spec, tensors)
    quant = evaluate.train_step(spec, tensors, quant=True)
    s, loss, st = run(spec, tensors, flags=L.abi.X_KEEP_ALL)
    print(name, "loss", loss, "oracle", exact["loss"], "oracle(bf16 storage)", quant["loss"], "kernels", st.n_kernels)
    assert abs(loss - quant["loss"]) <= TOL * abs(quant["loss"])
    assert abs(loss - exact["loss"]) <= TOL * abs(exact["loss"])
    got = {L_["name"]: s.activation(L_["name"]) for L_ in spec["layers"]}
    got.update(s.grads())
    wq, we = {}, {}
    for k, v in got.items():
        assert v.shape == exact[k].shape, k
        assert np.isfinite(v).all(), k
        wq[k] = rel_err(v, quant[k])
        we[k] = rel_err(v, exact[k])
    print("worst vs bf16-storage oracle:", sorted(wq.items(), key=lambda kv: -kv[1])[:4])
    print("worst vs exact oracle:", sorted(we.items(), key=lambda kv: -kv[1])[:4])
    if name not in DEEP:
        # The same gate with every backward activation gradient rounded where it is produced, whether the library
        # fuses it into a later sum / mask or not: where the backward roundings sit must not matter at this bound.
        from quant_marks import run_with_marks
        allb = run_with_marks(spec, tensors, "all_backward")
        wa = {k: rel_err(v, allb[k]) for k, v in got.items()}
        assert not {k: v for k, v in wa.items() if not v <= TOL}, wa
        # Against the oracle that never rounds, a parameter gradient may be off by what bf16 storage of the
        # activations alone costs (measured with the oracle: tests/test_oracle_quant.py) plus the bound itself.
        for k in (k for k in got if k.startswith("grad/")):
            storage = rel_err(quant[k], exact[k])
            assert we[k] <= TOL + storage * 1.01 + 1e-12, (k, we[k], storage)
            if name.startswith(("cfg1", "cfg2")):       # the two configured shallow workloads: 1.1e-2 and 4.2e-2 from storage alone
                assert we[k] <= 6e-2, (k, we[k])
    if name in DEEP:
        # one-ulp bf16 differences (fp32 against fp64 accumulation next to a rounding boundary) flip ReLU
        # decisions in the small late stages and are amplified from there: end to end only the loss and
        # the forward tensors are held to a bound, the sharp check is the per-node test below
        assert not {k: v for k, v in wq.items() if not k.startswith("grad/") and not v <= 2 * TOL}
    else:
        assert not {k: v for k, v in wq.items() if not v <= TOL}
        assert not {k: v for k, v in we.items() if not k.startswith("grad/") and not v <= TOL}


@pytest.mark.parametrize("name", list(SPECS))
def test_every_node_matches_oracle_on_its_own_inputs(name):
    """Every operation of the run (forward and backward) against the oracle's arithmetic applied to
    the inputs the GPU itself used: bf16 outputs within 1e-2 of the tensor's largest magnitude (one
    bf16 rounding is 2^-8 of an element), fp32 outputs (weight gradients, reductions) within 1e-4."""
    import paper_1807_02037_amd as L
    from node_oracle import eval_node
    A = L.abi
    spec = SPECS[name]()
    tensors = W.make_tensors(spec, affine="random")
    s, loss, st = run(spec, tensors, flags=A.X_KEEP_ALL)
    val = {}

    def value(i):
        if i not in val:
            val[i] = s.node_value(i)
        return val[i]
    worst = []
    for info in s.infos:
        if info.is_variable:
            continue
        shape = tuple(info.dims[i] for i in range(info.ndim))
        ref = eval_node(info, s.g.node_attr(info.id), [value(i) for i in s.g.node_inputs(info.id)], shape)
        got = value(info.id)
        assert got.shape == ref.shape and np.isfinite(got).all(), info.name
        tol = TOL if info.dtype == A.BF16 else 1e-4
        e = rel_err(got, ref)
        worst.append((e / tol, info.name.decode(), e))
        assert e <= tol, (info.name, e)
    print("closest to the bound:", sorted(worst, reverse=True)[:3])


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("mode", ["all_chain_rule", "all_fused_direct", "half_budget_own", "branches"])
def test_swapped_run_is_bit_identical(name, mode):
    import paper_1807_02037_amd as L
    A = L.abi
    spec = SPECS[name]()
    tensors = W.make_tensors(spec, affine="random")
    base, loss0, st0 = run(spec, tensors)
    g0 = base.grad_bits()
    if mode == "all_chain_rule":
        rw = dict()
    elif mode == "all_fused_direct":
        rw = dict(fuse_swapins=1, ctrld_strategy=A.DIRECT_ORDER, lb=2)
    elif mode == "branches":
        rw = dict(swap_branches=1, branch_threshold=2, fuse_swapins=1, lb=2)
    else:
        g, _ = L.build_graph(spec)
        need = g.memory_need()[1]
        floor = g.rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
        rw = dict(budget_bytes=(need + 2 * floor) // 3, fuse_swapins=1, ctrld_strategy=A.OWN)
    for flags in (0, A.X_POISON, A.X_NO_OVERLAP, A.X_ENCODE_SWAPS, A.X_ENCODE_SWAPS | A.X_POISON):
        s, loss, st = run(spec, tensors, rewrite=rw, flags=flags, steps=2)
        assert s.rewrite_stats.tensors_swapped > 0 and st.n_copies == s.rewrite_stats.swap_outs + s.rewrite_stats.swap_ins
        if flags & A.X_ENCODE_SWAPS:      # bitmap + non-zero values instead of the plain tensor: at most 1/16 + 1/2048 more
            assert 0 < st.bytes_d2h <= 1.07 * s.rewrite_stats.swapped_bytes_out + 4096 * s.rewrite_stats.swap_outs
            assert 0 < st.bytes_h2d <= 1.07 * s.rewrite_stats.swapped_bytes_in + 4096 * s.rewrite_stats.swap_ins
        else:
            assert st.bytes_d2h == s.rewrite_stats.swapped_bytes_out and st.bytes_h2d == s.rewrite_stats.swapped_bytes_in
        if "budget_bytes" in rw:
            assert s.arena_bytes <= rw["budget_bytes"] < base.arena_bytes
        assert np.float32(loss).view(np.uint32) == np.float32(loss0).view(np.uint32), (mode, flags)
        g1 = s.grad_bits()
        for k in g0:
            assert np.array_equal(g0[k], g1[k]), (mode, flags, k)


@pytest.mark.parametrize("name", ["pool_net", "cfg3_resnet_small", "cfg4_unet_small", "cfg2_stage_small", "updown_net"])
def test_recomputed_run_is_bit_identical(name):
    """Recomputation (Section 7, future work) combined with swapping: copies of cheap operations (mode 1), or chains
    of copies of any forward operation up to a depth, or the tensors the hybrid planner picks under a budget
    (mode 2), run again late instead of their outputs being swapped; no bit of the loss or of a gradient may change,
    also with released blocks poisoned and with only the copies (no swaps)."""
    import paper_1807_02037_amd as L
    A = L.abi
    spec = SPECS[name]()
    tensors = W.make_tensors(spec, affine="random")
    base, loss0, st0 = run(spec, tensors)
    g0 = base.grad_bits()
    floor = base.g.clone().rewrite(fuse_swapins=1, ctrld_strategy=A.OWN).arena_needed_after
    hybrid_budget = (base.unswapped_need + 3 * floor) // 4
    modes = [dict(recompute=2, recompute_depth=1, fuse_swapins=1), dict(recompute=2, recompute_depth=2, lb=2),
             dict(recompute=2, recompute_depth=3, ctrld_strategy=A.DIRECT_ORDER), dict(recompute=2, recompute_depth=50, n_tensors=0),
             dict(recompute=2, budget_bytes=hybrid_budget, fuse_swapins=1, ctrld_strategy=A.OWN)]
    if name in ("pool_net", "cfg3_resnet_small", "cfg4_unet_small"):      # nets with pooling / concatenation
        modes += [dict(recompute=1, fuse_swapins=1, lb=2), dict(recompute=1, n_tensors=0), dict(recompute=1, ctrld_strategy=A.DIRECT_ORDER)]
    for rw in modes:
        for flags in (A.X_POISON, A.X_ENCODE_SWAPS | A.X_POISON):
            s, loss, st = run(spec, tensors, rewrite=rw, flags=flags, steps=2)
            rs = s.rewrite_stats
            print(name, rw, "recomputed", rs.recomputed, "swapped", rs.tensors_swapped, "kernels", st.n_kernels, "vs", st0.n_kernels)
            # the planner under a budget may find that no recomputation pays on these tiny tensors
            assert (rs.recomputed > 0 or "budget_bytes" in rw) and st.n_copies == rs.swap_outs + rs.swap_ins
            assert st.n_kernels >= st0.n_kernels + rs.recomputed
            if rw.get("n_tensors") == 0:
                assert rs.tensors_swapped == 0 and st.n_copies == 0
            assert np.float32(loss).view(np.uint32) == np.float32(loss0).view(np.uint32), (rw, flags)
            g1 = s.grad_bits()
            for k in g0:
                assert np.array_equal(g0[k], g1[k]), (rw, flags, k)


def test_stream_timing_of_a_swapping_step():
    """LMS_X_TIMING: the step statistics say how long the compute stream stood waiting for swap-ins and swap-outs and
    how long the copy streams were busy; without the flag, and without swaps, the fields are zero."""
    import paper_1807_02037_amd as L
    A = L.abi
    spec = W.bottleneck_stage(batch=16, size=56)
    tensors = W.make_tensors(spec)
    rw = dict(n_tensors=-1, fuse_swapins=1)
    s0, loss0, st0 = run(spec, tensors, rewrite=rw, steps=2)
    for k in ("stall_h2d_ms", "stall_d2h_ms", "busy_d2h_ms", "busy_h2d_ms", "device_ms"):
        assert getattr(st0, k) == 0.0
    s1, loss1, st1 = run(spec, tensors, rewrite=rw, flags=A.X_TIMING, steps=3)
    assert np.float32(loss0).view(np.uint32) == np.float32(loss1).view(np.uint32)
    assert st1.n_copies == 2 * s1.rewrite_stats.tensors_swapped > 0
    assert 0.0 < st1.device_ms <= st1.ms * 1.05
    moved = s1.rewrite_stats.swapped_bytes_out
    for busy in (st1.busy_d2h_ms, st1.busy_h2d_ms):
        assert 0.0 < busy <= st1.device_ms * 1.05
        assert 5.0 < moved / busy / 1e6 < 70.0                    # GB/s over a PCIe Gen5 x16 link while busy
    # everything is swapped with the trigger one layer ahead: the backward pass waits for most of the swap-in time
    assert 0.0 < st1.stall_h2d_ms <= st1.device_ms and 0.0 <= st1.stall_d2h_ms <= st1.device_ms
    assert st1.stall_h2d_ms + st1.stall_d2h_ms >= 0.3 * (st1.device_ms - 1.5)
    s2, _, st2 = run(spec, tensors, flags=A.X_TIMING, steps=2)                # no swaps: nothing to wait for
    assert st2.stall_h2d_ms == 0.0 and st2.busy_d2h_ms == 0.0 and st2.device_ms > 0.0


def test_inference_graph_with_swapped_branches():
    """Forward-only graphs (Section 5.1, swap_branches for inference): the skip connections of the encoder-decoder
    are forward-to-forward edges longer than the threshold; swapping them must not change a bit of the output."""
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.unet3d(batch=1, size=16, base=32, levels=4, classes=4, cin=1)
    tensors = W.make_tensors(spec)
    base = Session(spec, tensors, backward=False, flags=A.X_KEEP_ALL)
    loss0, _ = base.step()
    out0 = base.activation(spec["loss"]["in"])
    none = Session(spec, tensors, backward=False, rewrite=dict(fuse_swapins=1))
    assert none.rewrite_stats.tensors_swapped == 0              # no backward phase: nothing to swap without branches
    for flags in (A.X_POISON, A.X_ENCODE_SWAPS | A.X_POISON):
        sw = Session(spec, tensors, backward=False, rewrite=dict(swap_branches=1, branch_threshold=3, fuse_swapins=1), flags=flags)
        assert sw.rewrite_stats.tensors_swapped == 3            # the three skip tensors
        assert sw.arena_bytes < base.unswapped_need
        for _ in range(2):
            loss1, st = sw.step()
        assert st.n_copies == 6
        assert np.float32(loss1).view(np.uint32) == np.float32(loss0).view(np.uint32)
    # the value of the output layer itself, with everything kept
    keep = Session(spec, tensors, backward=False, rewrite=dict(swap_branches=1, branch_threshold=3, fuse_swapins=1), flags=A.X_KEEP_ALL)
    keep.step()
    assert np.array_equal(keep.activation(spec["loss"]["in"]), out0)


def test_cfg1_budget_forces_exactly_two_swaps():
    import paper_1807_02037_amd as L
    spec = W.tiny_chain()
    tensors = W.make_tensors(spec)
    needs = []
    for n in range(3):
        g, _ = L.build_graph(spec)
        g.rewrite(n_tensors=n, fuse_swapins=1)
        needs.append(g.memory_need()[1])
    assert needs[2] < needs[1]
    s, loss, st = run(spec, tensors, rewrite=dict(budget_bytes=needs[2], fuse_swapins=1))
    assert s.rewrite_stats.tensors_swapped == 2 and st.n_copies == 4 and s.arena_bytes <= needs[2]
    ref = evaluate.train_step(spec, tensors, quant=True)
    assert abs(loss - ref["loss"]) <= TOL * abs(ref["loss"])
    for gname, gval in s.grads().items():
        assert rel_err(gval, ref[gname]) <= TOL, gname


def test_arena_too_small_is_an_error():
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    spec = W.tiny_chain()
    tensors = W.make_tensors(spec)
    with pytest.raises(L.LmsError) as e:
        Session(spec, tensors, arena_bytes=64 * 1024)
    assert e.value.status == L.abi.EOOM_DEVICE


def test_pinned_pool_of_the_library_is_device_visible_and_exact():
    """lms_pinned_alloc gives page-locked memory a kernel reads and writes at the host address: a plain swap copy
    (lms_device_copy) out to it and back returns every byte; the host sees what the device wrote."""
    import ctypes as C
    import numpy as np
    import torch
    from paper_1807_02037_amd import abi as A
    from paper_1807_02037_amd.api import PinnedPool
    n = 3 * 4096 + 16 * 5                                # not a power of two, not a page multiple
    pool = PinnedPool(n)
    assert pool.ptr % 4096 == 0 and pool.nbytes == n
    src = torch.arange(n, dtype=torch.int64, device="cuda").mul_(37).to(torch.uint8)
    back = torch.zeros(n, dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    assert A.lib().lms_device_copy(pool.ptr, src.data_ptr(), n, s) == A.OK
    torch.cuda.synchronize()
    host = np.ctypeslib.as_array((C.c_uint8 * n).from_address(pool.ptr)).copy()
    assert np.array_equal(host, src.cpu().numpy())
    assert A.lib().lms_device_copy(back.data_ptr(), pool.ptr, n, s) == A.OK
    torch.cuda.synchronize()
    assert torch.equal(back, src)
    pool.free()
    pool.free()                                          # a second call is a no-op
