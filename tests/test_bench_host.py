"""Host-side helpers of bench.py: the searches for the largest batch under a cap are planner work only."""
import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import bench  # noqa: E402
import workloads as W  # noqa: E402
from paper_1807_02037_amd import abi as A  # noqa: E402
from paper_1807_02037_amd.api import LmsError  # noqa: E402
from paper_1807_02037_amd.models import build_graph  # noqa: E402

CAP = 2 * 10**9          # a small cap keeps the graphs of the search small
SIZE = 64


def make(b):
    return W.resnet50(batch=b, size=SIZE)


def need(b, **kw):
    g = build_graph(make(b))[0]
    if kw:
        g.rewrite(**kw)
    return g.memory_need()[1]


def test_largest_unswapped_batch_is_the_last_that_fits():
    b0 = bench.largest_unswapped_batch(CAP, SIZE)
    assert b0 > 0 and need(b0) <= CAP < need(b0 + 1)


@pytest.mark.parametrize("kw", [dict(n_tensors=-1, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1),
                                dict(n_tensors=12, lb=1, ctrld_strategy=A.CHAIN_RULE, fuse_swapins=1),
                                dict(n_tensors=-1, lb=5, ctrld_strategy=A.DIRECT_ORDER, fuse_swapins=0)])
def test_largest_batch_of_a_fixed_setting_is_the_last_whose_plan_fits(kw):
    b = bench.largest_batch_with_setting(CAP, make, kw)
    assert b > bench.largest_unswapped_batch(CAP, SIZE)          # swapping buys batch
    assert need(b, **kw) <= CAP < need(b + 1, **kw)


def test_a_setting_with_a_budget_is_given_the_cap_and_agrees_with_the_headline_search():
    kw = dict(ctrld_strategy=A.OWN, fuse_swapins=1, budget_bytes=12345)
    b = bench.largest_batch_with_setting(CAP, make, kw)
    assert b == bench.largest_swapped_batch(CAP, SIZE, 1, bench.rewrite_kw(0, encoded=False))
    build_graph(make(b))[0].rewrite(budget_bytes=CAP, ctrld_strategy=A.OWN, fuse_swapins=1)
    with pytest.raises(LmsError):
        build_graph(make(b + 1))[0].rewrite(budget_bytes=CAP, ctrld_strategy=A.OWN, fuse_swapins=1)


def test_sweep_settings_cover_table_2():
    st = bench.sweep_settings(make(4))
    keys = set().union(*[set(s) for s in st])
    assert {"n_tensors", "lb", "ctrld_strategy", "fuse_swapins", "swap_branches", "branch_threshold", "budget_bytes"} <= keys
    assert {s["ctrld_strategy"] for s in st} == {A.CHAIN_RULE, A.DIRECT_ORDER, A.OWN}
    assert {s.get("lb") for s in st} >= {1, 5, 20, 100}
