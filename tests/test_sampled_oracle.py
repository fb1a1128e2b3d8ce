"""The sampled checker used at full size (tests/sampled_oracle.py) against the whole-tensor oracle on small
geometries: the sampled values must be the oracle's values at the sampled places, the checker must compare at
least 4096 elements per node where the node has that many, and a planted mistake in one output tile must be found."""
from types import SimpleNamespace

import numpy as np
import pytest

import workloads as W
from oracle import ops
from paper_1807_02037_amd import abi as A
import sampled_oracle as S

GEOMS = [
    # n, in_sp, c, k, filt, stride, pad
    (3, (9, 11), 8, 16, (3, 3), 1, 1),
    (2, (15, 17), 16, 8, (3, 3), 2, 1),
    (2, (14, 14), 24, 40, (1, 1), 1, 0),
    (2, (16, 16), 8, 24, (1, 1), 2, 0),
    (1, (20, 20), 3, 16, (7, 7), 2, 3),
    (1, (6, 7, 9), 8, 16, (3, 3, 3), 1, 1),
    (2, (6, 6, 6), 8, 8, (2, 2, 2), 2, 0),
]


def _data(seed, n, in_sp, c, k, filt, stride, pad):
    x = W.round_to_bf16(W.normal(seed, (n,) + in_sp + (c,)))
    w = W.round_to_bf16(W.normal(seed + 1, filt + (c, k), 0.2))
    y = ops.conv_fwd(x, w, stride, pad)
    dy = W.round_to_bf16(W.normal(seed + 2, y.shape))
    return x, w, y, dy


@pytest.mark.parametrize("geom", GEOMS, ids=[str(g) for g in GEOMS])
def test_sampled_values_are_the_oracle_values(geom):
    n, in_sp, c, k, filt, stride, pad = geom
    x, w, y, dy = _data(500, *geom)
    rng = np.random.default_rng(3)
    pos = S.sample_positions(rng, y.shape[:-1], 50)
    assert np.allclose(S.conv_fwd_at(x, w, stride, pad, pos), y[tuple(pos.T)], rtol=0, atol=1e-11)
    dx = ops.conv_dgrad(dy, w, x.shape, stride, pad)
    pos = S.sample_positions(rng, x.shape[:-1], 50)
    assert np.allclose(S.conv_dgrad_at(dy, w, stride, pad, pos), dx[tuple(pos.T)], rtol=0, atol=1e-11)
    dw = ops.conv_wgrad(x, dy, filt, stride, pad)
    for tap in S.sample_taps(rng, filt, c, k):
        for chunk in (None, 1):
            assert np.allclose(S.conv_wgrad_tap(x, dy, stride, pad, tap, chunk), dw[tap], rtol=0, atol=1e-10)


def _node(op, flags=0, stride=1, pad=0):
    return SimpleNamespace(op=op), SimpleNamespace(flags=flags, stride=stride, pad=pad)


def test_checker_covers_every_op_and_counts_enough_elements():
    rng = np.random.default_rng(11)
    n, in_sp, c, k, filt, stride, pad = 2, (20, 20), 16, 32, (3, 3), 1, 1
    x, w, y, dy = _data(900, n, in_sp, c, k, filt, stride, pad)
    scale = 1.0 + 0.1 * W.normal(77, (k,)).astype(np.float32).astype(np.float64)
    shift = 0.1 * W.normal(78, (k,)).astype(np.float32).astype(np.float64)
    res = W.round_to_bf16(W.normal(79, y.shape))
    out = ops.relu(ops.affine_fwd(y, scale, shift) + res)
    info, attr = _node(A.OP_CONV, A.F_AFFINE | A.F_RES | A.F_RELU, stride, pad)
    e, cnt = S.check_conv_node(rng, info, attr, [x, w, scale, shift, res], out)
    assert e < 1e-12 and cnt >= S.MIN_ELEMENTS
    mask = W.round_to_bf16(W.normal(80, x.shape))
    add = W.round_to_bf16(W.normal(81, x.shape))
    info, attr = _node(A.OP_CONV_DGRAD, A.F_ADDEND | A.F_MASK, stride, pad)
    dx = ops.relu_grad(ops.conv_dgrad(dy, w, x.shape, stride, pad) + add, mask)
    e, cnt = S.check_conv_node(rng, info, attr, [dy, w, add, mask], dx)
    assert e < 1e-12 and cnt >= S.MIN_ELEMENTS
    info, attr = _node(A.OP_CONV_WGRAD, 0, stride, pad)
    e, cnt = S.check_conv_node(rng, info, attr, [x, dy], ops.conv_wgrad(x, dy, filt, stride, pad))
    assert e < 1e-12 and cnt >= S.MIN_ELEMENTS
    # transposed convolution, window = stride = 2
    xs = W.round_to_bf16(W.normal(82, (2, 6, 7, 16)))
    wt = W.round_to_bf16(W.normal(83, (2, 2, 16, 32), 0.2))
    yt = ops.tconv_fwd(xs, wt)
    dyt = W.round_to_bf16(W.normal(84, yt.shape))
    info, attr = _node(A.OP_TCONV)
    e, cnt = S.check_conv_node(rng, info, attr, [xs, wt], yt)
    assert e < 1e-12 and cnt >= min(S.MIN_ELEMENTS, yt.size)
    info, attr = _node(A.OP_TCONV_DGRAD)
    e, cnt = S.check_conv_node(rng, info, attr, [dyt, wt], ops.tconv_dgrad(dyt, wt))
    assert e < 1e-12 and cnt >= min(S.MIN_ELEMENTS, xs.size)
    info, attr = _node(A.OP_TCONV_WGRAD)
    e, cnt = S.check_conv_node(rng, info, attr, [xs, dyt], ops.tconv_wgrad(xs, dyt))
    assert e < 1e-12 and cnt == wt.size


def test_a_wrong_partial_filter_or_tile_is_found():
    """Planted mistakes (in the oracle-side copy of the output): one tap slice of a weight gradient off by the
    contribution of one split, and one 8-channel vector of a forward output."""
    n, in_sp, c, k, filt, stride, pad = 2, (20, 20), 16, 32, (3, 3), 1, 1
    x, w, y, dy = _data(901, n, in_sp, c, k, filt, stride, pad)
    dw = ops.conv_wgrad(x, dy, filt, stride, pad)
    bad = dw.copy()
    bad[0, 0] += ops.conv_wgrad(x[:1, :4], dy[:1, :4], filt, stride, pad)[0, 0] * 0.5   # a fraction of one split
    info, attr = _node(A.OP_CONV_WGRAD, 0, stride, pad)
    e, _ = S.check_conv_node(np.random.default_rng(5), info, attr, [x, dy], bad)
    assert e > 1e-4
    info, attr = _node(A.OP_CONV, 0, stride, pad)
    hits = 0
    for seed in range(20):
        bad = y.copy()
        r = np.random.default_rng(100 + seed)
        p = tuple(int(r.integers(0, d)) for d in y.shape[:-1])
        bad[p][8:16] += 0.05 * np.abs(y).max()
        e, _ = S.check_conv_node(np.random.default_rng(seed), info, attr, [x, w], bad)
        hits += e > 1e-2
    # 128 + 4 of 800 positions are sampled: a single wrong position is seen about one time in six, a wrong
    # 128-position tile always
    assert 1 <= hits <= 12
    bad = y.copy()
    bad[0, :8, :16, 8:16] += 0.05 * np.abs(y).max()
    e, _ = S.check_conv_node(np.random.default_rng(1), info, attr, [x, w], bad)
    assert e > 1e-2
