"""Parity at the full sizes of the configured workloads, in the launch configuration the benchmark times.

A whole fp64 oracle step is too slow there, so every node of a GPU run is checked on its own inputs:
convolution-type nodes on sampled output elements recomputed one by one from the definition, all other
nodes (element-wise, pooling, losses, reductions) in full with the oracle's arithmetic.  The swapping run
(budget = half the footprint, fused swap-ins, budget-driven placement: what bench.py times) must then be
bit-identical to the unswapped run, so the sampled checks carry over to it."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def check_all_nodes(spec, tensors, samples=40):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    from node_oracle import eval_node
    from sampled_oracle import check_conv_node, CONV_OPS
    A = L.abi
    s = Session(spec, tensors, flags=A.X_KEEP_ALL)
    loss, st = s.step()
    assert np.isfinite(loss)
    rng = np.random.default_rng(1807)
    cache = {}
    last_reader = {}
    for info in s.infos:
        for i in s.g.node_inputs(info.id):
            last_reader[i] = info.id

    def value(i):
        if i not in cache:
            cache[i] = s.node_value(i)
        return cache[i]
    worst = []
    for info in s.infos:
        if info.is_variable:
            continue
        ins = [value(i) for i in s.g.node_inputs(info.id)]
        got = value(info.id)
        assert np.isfinite(got).all(), info.name
        tol = 1e-2 if info.dtype == A.BF16 else 1e-4
        if info.op in CONV_OPS:
            e = check_conv_node(rng, info, s.g.node_attr(info.id), ins, got, samples)
        else:
            shape = tuple(info.dims[i] for i in range(info.ndim))
            ref = eval_node(info, s.g.node_attr(info.id), ins, shape)
            e = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)
        worst.append((e / tol, info.name.decode(), e))
        assert e <= tol, (info.name, e)
        # drop values nobody needs any more (keeps host memory bounded)
        for i in list(cache):
            if last_reader.get(i, -1) <= info.id:
                del cache[i]
    print("closest to the bound:", sorted(worst, reverse=True)[:4])
    return s, loss


def test_config2_full_size_nodes_and_swapped_bit_identity():
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = W.bottleneck_stage()
    tensors = W.make_tensors(spec)
    s0, loss0 = check_all_nodes(spec, tensors)
    g0 = s0.grad_bits()
    del s0
    base = Session(spec, tensors)
    loss_b, _ = base.step()
    gb = base.grad_bits()
    footprint = base.unswapped_need
    del base
    sw = Session(spec, tensors, rewrite=dict(budget_bytes=footprint // 2, fuse_swapins=1, ctrld_strategy=A.OWN))
    for _ in range(2):
        loss_s, st = sw.step()
    assert sw.arena_bytes <= footprint // 2 and st.n_copies == 2 * sw.rewrite_stats.tensors_swapped > 0
    gs = sw.grad_bits()
    for a, b in ((loss0, loss_b), (loss_b, loss_s)):
        assert np.float32(a).view(np.uint32) == np.float32(b).view(np.uint32)
    for k in g0:
        assert np.array_equal(g0[k], gb[k]) and np.array_equal(gb[k], gs[k]), k


def test_config4_unet_128_nodes():
    spec = W.unet3d(batch=1, size=128)
    tensors = W.make_tensors(spec)
    check_all_nodes(spec, tensors, samples=24)


def test_config3_resnet50_224_nodes():
    spec = W.resnet50(batch=8, size=224)
    tensors = W.make_tensors(spec, affine="random")
    check_all_nodes(spec, tensors, samples=16)
