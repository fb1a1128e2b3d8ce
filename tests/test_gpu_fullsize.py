"""Parity at the full sizes of the configured workloads, in the launch configuration the benchmark times.

A whole fp64 oracle step is too slow there, so every node of a GPU run is checked on its own inputs:
convolution-type nodes on at least 4096 sampled output elements recomputed from the definition (whole filter taps
for weight gradients), all other nodes (element-wise, pooling, losses, reductions) in full with the oracle's
arithmetic.  A run that swaps under a cap (fused swap-ins, budget-driven placement: what bench.py times) must then
be bit-identical to the unswapped run in its loss and in every parameter gradient, so the sampled checks carry over
to it (swap operations are identities, Eq. 2 / Eq. 5)."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def check_all_nodes(spec, tensors, samples=40):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    from node_oracle import eval_node
    from sampled_oracle import check_conv_node, CONV_OPS, MIN_ELEMENTS
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
        tol = 1e-2 if info.dtype == A.BF16 else 1e-4
        if info.op in CONV_OPS:
            # sampled on the device tensors: only the sampled rows (or one batch chunk) come to the host
            ins = [s.node_tensor(i) for i in s.g.node_inputs(info.id)]
            got = s.node_tensor(info.id)
            e, count = check_conv_node(rng, info, s.g.node_attr(info.id), ins, got, samples)
            assert count >= min(MIN_ELEMENTS, got.numel()), (info.name, count)
        else:
            ins = [value(i) for i in s.g.node_inputs(info.id)]
            got = value(info.id)
            assert np.isfinite(got).all(), info.name
            shape = tuple(info.dims[i] for i in range(info.ndim))
            ref = eval_node(info, s.g.node_attr(info.id), ins, shape)
            e = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)
        assert np.isfinite(e), info.name
        worst.append((e / tol, info.name.decode(), e))
        assert e <= tol, (info.name, e)
        # drop values nobody needs any more (keeps host memory bounded)
        for i in list(cache):
            if last_reader.get(i, -1) <= info.id:
                del cache[i]
    print("closest to the bound:", sorted(worst, reverse=True)[:4])
    return s, loss


def same_bits(a, b):
    return np.float32(a).view(np.uint32) == np.float32(b).view(np.uint32)


def assert_swapped_equals_unswapped(spec, tensors, budget_of, flags=0, steps=2, grads_ref=None, loss_ref=None, recompute=0):
    """Runs the workload unswapped, then rewritten for budget_of(unswapped footprint), and compares the loss and
    every parameter gradient bit for bit.  Returns the swapping session's rewrite statistics."""
    import torch
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    base = Session(spec, tensors)
    loss_b, _ = base.step()
    gb = base.grad_bits()
    footprint = base.unswapped_need
    del base
    torch.cuda.empty_cache()
    if loss_ref is not None:
        assert same_bits(loss_ref, loss_b)
        for k in grads_ref:
            assert np.array_equal(grads_ref[k], gb[k]), k
    budget = int(budget_of(footprint))
    sw = Session(spec, tensors, rewrite=dict(budget_bytes=budget, fuse_swapins=1, ctrld_strategy=A.OWN, recompute=recompute),
                 flags=flags)
    for _ in range(steps):
        loss_s, st = sw.step()
    rs = sw.rewrite_stats
    assert sw.arena_bytes <= budget and rs.tensors_swapped + rs.recomputed > 0 and st.n_copies == rs.swap_outs + rs.swap_ins
    assert (rs.recomputed > 0) == (recompute > 0)
    gs = sw.grad_bits()
    assert same_bits(loss_b, loss_s)
    assert len(gs) == len(gb) > 0
    for k in gb:
        assert np.array_equal(gb[k], gs[k]), k
    del sw
    torch.cuda.empty_cache()
    return rs


def test_config2_full_size_nodes_and_swapped_bit_identity():
    spec = W.bottleneck_stage()
    tensors = W.make_tensors(spec)
    s0, loss0 = check_all_nodes(spec, tensors)
    g0 = s0.grad_bits()
    del s0
    rs = assert_swapped_equals_unswapped(spec, tensors, lambda fp: fp // 2, grads_ref=g0, loss_ref=loss0)
    assert rs.swap_ins == rs.swap_outs


def test_config4_unet_128_nodes_and_swapped_bit_identity():
    import paper_1807_02037_amd as L
    spec = W.unet3d(batch=1, size=128)
    tensors = W.make_tensors(spec)
    s0, loss0 = check_all_nodes(spec, tensors, samples=24)
    g0 = s0.grad_bits()
    del s0
    assert_swapped_equals_unswapped(spec, tensors, lambda fp: fp // 2, grads_ref=g0, loss_ref=loss0)
    assert_swapped_equals_unswapped(spec, tensors, lambda fp: fp // 2, flags=L.abi.X_ENCODE_SWAPS)
    # the hybrid planner (per tensor recompute / swap / keep) under the same half-footprint budget
    rs = assert_swapped_equals_unswapped(spec, tensors, lambda fp: fp // 2, flags=L.abi.X_ENCODE_SWAPS, recompute=2)
    assert rs.recomputed >= 4


def test_config5_unet_192_nodes_and_swapped_bit_identity():
    """3-D U-Net at 192^3, batch 1: every node against the oracle on its own inputs, then the run under half the
    unswapped footprint (the 16 GB cap of the configuration forces no swapping in bf16) against the unswapped run."""
    from bench import device_tensors
    spec = W.unet3d(batch=1, size=192)
    tensors = W.make_tensors(spec)
    s0, loss0 = check_all_nodes(spec, tensors, samples=24)
    g0 = s0.grad_bits()
    del s0
    assert_swapped_equals_unswapped(spec, tensors, lambda fp: fp // 2, grads_ref=g0, loss_ref=loss0)
    # batch 2 of the same configuration: swapped against unswapped only (the nodes are the batch-1 kernels)
    spec2 = W.unet3d(batch=2, size=192)
    assert_swapped_equals_unswapped(spec2, device_tensors(spec2, 1), lambda fp: fp // 2, steps=1)


def test_config3_resnet50_224_nodes():
    spec = W.resnet50(batch=8, size=224)
    tensors = W.make_tensors(spec, affine="random")
    check_all_nodes(spec, tensors, samples=16)


def test_config3_resnet50_224_swapped_bit_identity_under_16gb():
    """ResNet-50 at 224x224 and 1.5 times the largest batch that fits 16 GB unswapped: the rewritten plan under the
    16 GB cap against the uncapped run, loss and all 161 parameter gradients, plain and encoded swap copies."""
    import paper_1807_02037_amd as L
    from bench import device_tensors
    spec = W.resnet50(batch=1276, size=224)
    tensors = device_tensors(spec, 8)
    cap = 16 * 10 ** 9
    rs = assert_swapped_equals_unswapped(spec, tensors, lambda fp: cap)
    assert rs.tensors_swapped >= 5
    assert_swapped_equals_unswapped(spec, tensors, lambda fp: cap, flags=L.abi.X_ENCODE_SWAPS, steps=1)
    rs2 = assert_swapped_equals_unswapped(spec, tensors, lambda fp: cap, flags=L.abi.X_ENCODE_SWAPS, steps=1, recompute=2)
    assert rs2.swapped_bytes_out < rs.swapped_bytes_out
