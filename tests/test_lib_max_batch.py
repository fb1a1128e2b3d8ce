"""The metric's 'maximum batch under the device-memory cap' is host logic: the planner's footprint of ResNet-50 224x224
without swapping, and the rewriter's verdict with every eligible tensor allowed to swap.  Pins the two batches the
measurements are quoted on (16 GB cap) and checks that each is the exact threshold."""
import workloads as W
import paper_1807_02037_amd as L
from paper_1807_02037_amd.models import build_graph

A = L.abi
CAP = 16 * 10 ** 9


def footprint(batch):
    return build_graph(W.resnet50(batch=batch, size=224))[0].memory_need()[1]


def rewritten_arena(batch):
    g = build_graph(W.resnet50(batch=batch, size=224))[0]
    g.rewrite(budget_bytes=CAP, fuse_swapins=1, ctrld_strategy=A.OWN)
    return g.memory_need()[1]


def test_largest_batch_without_swapping_is_852():
    assert footprint(852) <= CAP < footprint(853)
    # about 18.8 MB of activations per image (filters are bound variables outside the arena)
    assert 18.0e6 < (footprint(852) - footprint(752)) / 100 < 19.5e6


def test_largest_batch_with_swapping_is_3796():
    assert rewritten_arena(3796) <= CAP
    try:
        rewritten_arena(3797)
    except L.LmsError as e:
        assert "budget" in str(e)
    else:
        raise AssertionError("batch 3797 must not fit a 16 GB arena")
    assert 3796 / 852 > 4.4
