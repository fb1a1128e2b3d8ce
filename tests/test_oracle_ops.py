"""Pins of the oracle's layer arithmetic against things other than itself: brute-force
loops, library routines it reduces to in special cases, closed forms, adjoint identities
and central finite differences of whole training steps."""
import itertools
import math

import numpy as np
import pytest
from scipy import signal

import workloads as W
from oracle import ops, evaluate

RNG = np.random.default_rng(7)


def brute_conv(x, w, stride, pad):
    nd = x.ndim - 2
    N, sp, C = x.shape[0], x.shape[1:-1], x.shape[-1]
    filt, K = w.shape[:nd], w.shape[-1]
    osp = tuple((sp[i] + 2 * pad - filt[i]) // stride + 1 for i in range(nd))
    y = np.zeros((N,) + osp + (K,))
    for n in range(N):
        for o in itertools.product(*[range(s) for s in osp]):
            for k in range(K):
                acc = 0.0
                for r in itertools.product(*[range(f) for f in filt]):
                    pos = tuple(o[i] * stride + r[i] - pad for i in range(nd))
                    if any(p < 0 or p >= sp[i] for i, p in enumerate(pos)):
                        continue
                    for c in range(C):
                        acc += x[(n,) + pos + (c,)] * w[r + (c, k)]
                y[(n,) + o + (k,)] = acc
    return y


@pytest.mark.parametrize("shape,filt,stride,pad", [
    ((2, 5, 6, 3), (3, 3), 1, 1), ((1, 7, 7, 2), (3, 3), 2, 1), ((1, 6, 5, 2), (1, 1), 2, 0),
    ((1, 9, 8, 2), (7, 7), 2, 3), ((1, 4, 5, 3, 2), (3, 3, 3), 1, 1), ((1, 4, 4, 4, 2), (2, 2, 2), 2, 0),
])
def test_conv_fwd_brute_force(shape, filt, stride, pad):
    x = RNG.standard_normal(shape)
    w = RNG.standard_normal(filt + (shape[-1], 4))
    np.testing.assert_allclose(ops.conv_fwd(x, w, stride, pad), brute_conv(x, w, stride, pad), rtol=1e-12, atol=1e-12)


def test_conv_is_correlation_library():
    # single channel, no padding: the library's "valid" cross-correlation
    x = RNG.standard_normal((1, 9, 11, 1))
    w = RNG.standard_normal((3, 4, 1, 1))
    ref = signal.correlate(x[0, :, :, 0], w[:, :, 0, 0], mode="valid")
    np.testing.assert_allclose(ops.conv_fwd(x, w)[0, :, :, 0], ref, rtol=1e-12, atol=1e-12)
    x3 = RNG.standard_normal((1, 5, 6, 7, 1))
    w3 = RNG.standard_normal((3, 2, 3, 1, 1))
    ref3 = signal.correlate(x3[0, ..., 0], w3[..., 0, 0], mode="valid")
    np.testing.assert_allclose(ops.conv_fwd(x3, w3)[0, ..., 0], ref3, rtol=1e-12, atol=1e-12)


def test_conv_special_cases():
    x = RNG.standard_normal((2, 4, 5, 6))
    w = RNG.standard_normal((1, 1, 6, 3))
    # 1x1 stride 1 is a plain matrix product over channels
    np.testing.assert_allclose(ops.conv_fwd(x, w).reshape(-1, 3), x.reshape(-1, 6) @ w[0, 0], rtol=1e-13)
    # delta filter at tap (0, 2) of a 3x3, pad 1: output is the input shifted one column left
    d = np.zeros((3, 3, 6, 6))
    d[0, 2] = np.eye(6)
    y = ops.conv_fwd(x, d, 1, 1)
    np.testing.assert_array_equal(y[:, 1:, :-1], x[:, :-1, 1:])
    assert np.all(y[:, 0] == 0) and np.all(y[:, :, -1] == 0)
    # filter as large as the image, no padding: one dot product per (n, k)
    wf = RNG.standard_normal((4, 5, 6, 2))
    np.testing.assert_allclose(ops.conv_fwd(x, wf)[:, 0, 0], np.einsum("nhwc,hwck->nk", x, wf), rtol=1e-12)


@pytest.mark.parametrize("shape,filt,stride,pad", [
    ((2, 6, 7, 3), (3, 3), 1, 1), ((2, 7, 8, 3), (3, 3), 2, 1), ((1, 8, 8, 2), (1, 1), 2, 0),
    ((1, 11, 10, 2), (7, 7), 2, 3), ((1, 5, 4, 6, 2), (3, 3, 3), 1, 1),
])
def test_conv_adjoints(shape, filt, stride, pad):
    x = RNG.standard_normal(shape)
    w = RNG.standard_normal(filt + (shape[-1], 5))
    y = ops.conv_fwd(x, w, stride, pad)
    dy = RNG.standard_normal(y.shape)
    lhs = (y * dy).sum()
    assert math.isclose(lhs, (x * ops.conv_dgrad(dy, w, x.shape, stride, pad)).sum(), rel_tol=1e-11)
    assert math.isclose(lhs, (w * ops.conv_wgrad(x, dy, filt, stride, pad)).sum(), rel_tol=1e-11)


def test_tconv_is_adjoint_of_strided_conv():
    # a 2x2x2 stride-2 transposed convolution is the adjoint of a 2x2x2 stride-2 convolution
    x = RNG.standard_normal((2, 3, 2, 4, 5))
    w = RNG.standard_normal((2, 2, 2, 5, 3))          # (taps, C_in, C_out) of the transposed conv
    y = ops.tconv_fwd(x, w)
    assert y.shape == (2, 6, 4, 8, 3)
    wc = np.swapaxes(w, -1, -2)                        # the forward conv maps C_out -> C_in
    np.testing.assert_allclose(y, ops.conv_dgrad(x, wc, y.shape, 2, 0), rtol=1e-12, atol=1e-13)
    dy = RNG.standard_normal(y.shape)
    lhs = (y * dy).sum()
    assert math.isclose(lhs, (x * ops.tconv_dgrad(dy, w)).sum(), rel_tol=1e-11)
    assert math.isclose(lhs, (w * ops.tconv_wgrad(x, dy)).sum(), rel_tol=1e-11)
    # explicit element
    n, d, h, ww, k = 1, 2, 1, 3, 2
    ref = sum(x[n, d, h, ww, c] * w[1, 0, 1, c, k] for c in range(5))
    assert math.isclose(y[n, 2 * d + 1, 2 * h, 2 * ww + 1, k], ref, rel_tol=1e-12)


def test_relu_and_ties():
    y = np.array([-1.0, 0.0, 2.0])
    np.testing.assert_array_equal(ops.relu(y), [0.0, 0.0, 2.0])
    np.testing.assert_array_equal(ops.relu_grad(np.ones(3), ops.relu(y)), [0.0, 0.0, 1.0])


def test_maxpool_routing_and_ties():
    x = np.zeros((1, 4, 4, 1))
    x[0, :2, :2, 0] = [[3.0, 3.0], [3.0, 1.0]]       # three-way tie: first in row-major order wins
    x[0, 2:, 2:, 0] = [[-5.0, -2.0], [-2.0, -7.0]]   # all negative
    y, arg = ops.maxpool_fwd(x, 2, 2, 0)
    np.testing.assert_array_equal(y[0, :, :, 0], [[3.0, 0.0], [0.0, -2.0]])
    assert arg[0, 0, 0, 0] == 0 and arg[0, 1, 1, 0] == 1 and arg[0, 0, 1, 0] == 0
    dx = ops.maxpool_bwd(np.full((1, 2, 2, 1), 1.0), arg, x.shape, 2, 2, 0)
    expect = np.zeros((4, 4))
    expect[0, 0] = expect[0, 2] = expect[2, 0] = expect[2, 3] = 1.0
    np.testing.assert_array_equal(dx[0, :, :, 0], expect)
    # padded 3x3 stride 2: padding never wins, every gradient lands inside the image
    x2 = -np.abs(RNG.standard_normal((1, 5, 5, 2))) - 1.0
    y2, a2 = ops.maxpool_fwd(x2, 3, 2, 1)
    assert y2.shape == (1, 3, 3, 2) and np.all(y2 < 0)
    dx2 = ops.maxpool_bwd(np.ones(y2.shape), a2, x2.shape, 3, 2, 1)
    assert dx2.sum() == y2.size
    # brute-force value check
    for o in itertools.product(range(3), range(3)):
        win = x2[0, max(0, 2 * o[0] - 1):2 * o[0] + 2, max(0, 2 * o[1] - 1):2 * o[1] + 2, 0]
        assert y2[0, o[0], o[1], 0] == win.max()


def test_losses_closed_forms():
    for K in (4, 1000):
        z = np.full((3, K), 0.7)
        lab = np.array([0, K - 1, K // 2])
        assert math.isclose(ops.softmax_ce_fwd(z, lab), math.log(K), rel_tol=1e-12)
        dz = ops.softmax_ce_bwd(z, lab)
        np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-15)
        assert math.isclose(dz[0, 0], (1.0 / K - 1.0) / 3, rel_tol=1e-12)
        assert math.isclose(dz[0, 1], (1.0 / K) / 3, rel_tol=1e-12)
    # shift invariance and a large-logit case that would overflow without max subtraction
    z = RNG.standard_normal((2, 3, 5)) * 3
    lab = RNG.integers(0, 5, (2, 3))
    assert math.isclose(ops.softmax_ce_fwd(z, lab), ops.softmax_ce_fwd(z + 1000.0, lab), rel_tol=1e-10)
    # two-class case equals the logistic loss
    z2 = np.array([[1.5, -0.5]])
    assert math.isclose(ops.softmax_ce_fwd(z2, np.array([0])), math.log1p(math.exp(-2.0)), rel_tol=1e-12)
    y = RNG.standard_normal((2, 3, 4))
    assert ops.mse_fwd(y, y) == 0.0
    t = np.zeros_like(y)
    assert math.isclose(ops.mse_fwd(y, t), (y ** 2).mean(), rel_tol=1e-12)
    np.testing.assert_allclose(ops.mse_bwd(y, t), y / 12.0, rtol=1e-12)


def test_gap_affine_bias_concat():
    x = RNG.standard_normal((2, 3, 4, 5))
    np.testing.assert_allclose(ops.gap_fwd(x)[:, 0, 0], x.reshape(2, 12, 5).mean(axis=1), rtol=1e-12)
    assert math.isclose(ops.gap_bwd(np.ones((2, 1, 1, 5)), x.shape)[0, 0, 0, 0], 1 / 12.0)
    s, h = RNG.standard_normal(5), RNG.standard_normal(5)
    y = ops.affine_fwd(x, s, h)
    assert math.isclose(y[1, 2, 3, 4], s[4] * x[1, 2, 3, 4] + h[4])
    dy = RNG.standard_normal(x.shape)
    dx, ds, dh = ops.affine_bwd(dy, x, s)
    assert math.isclose(ds[2], (dy[..., 2] * x[..., 2]).sum(), rel_tol=1e-12)
    assert math.isclose(dh[2], dy[..., 2].sum(), rel_tol=1e-12)
    assert math.isclose(dx[0, 1, 2, 3], s[3] * dy[0, 1, 2, 3])
    a, b = RNG.standard_normal((1, 2, 2, 3)), RNG.standard_normal((1, 2, 2, 4))
    c = ops.concat(a, b)
    assert c.shape[-1] == 7 and np.all(c[..., :3] == a) and np.all(c[..., 3:] == b)
    da, db = ops.concat_bwd(c, 3)
    assert np.all(da == a) and np.all(db == b)


def _smooth_inputs(spec, seed):
    """Tensors for finite differences: generic fp64 values (no bf16 grid), affine/bias non-trivial."""
    t = W.make_tensors(spec, affine="random")
    r = np.random.default_rng(seed)
    for k, v in t.items():
        if v.dtype.kind == "f":
            t[k] = v + 0.01 * r.standard_normal(v.shape)
    return t


FD_SPECS = [
    ("tiny_chain", lambda: W.tiny_chain(batch=2, size=6, cin=3, width=4, depth=3, classes=3)),
    ("bottleneck", lambda: W.bottleneck_stage(batch=2, size=5, cin=8, width=4, blocks=2)),
    ("resnet", lambda: W.resnet50(batch=2, size=20, classes=5, stage_blocks=(1, 2), base=4)),
    ("unet3d", lambda: W.unet3d(batch=1, size=4, base=2, levels=2, classes=3, cin=1)),
    ("unet3d_deep", lambda: W.unet3d(batch=1, size=8, base=2, levels=3, classes=3, cin=2)),
]


@pytest.mark.parametrize("name,mk", FD_SPECS, ids=[s[0] for s in FD_SPECS])
def test_training_step_finite_differences(name, mk):
    """Central differences of the loss in a few entries of every parameter against the
    back-propagated gradients (ReLU / max-pool kinks are measure-zero for generic inputs)."""
    spec = mk()
    t = _smooth_inputs(spec, 11)
    base = evaluate.train_step(spec, t)
    r = np.random.default_rng(5)
    h = 1e-6
    checked = 0
    for pname in [k for k in t if "." in k]:
        g = base["grad/" + pname]
        assert g.shape == t[pname].shape
        flat = t[pname].reshape(-1)
        for idx in r.choice(flat.size, size=min(3, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            lp = evaluate.train_step(spec, t)["loss"]
            flat[idx] = old - h
            lm = evaluate.train_step(spec, t)["loss"]
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = g.reshape(-1)[idx]
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an), abs(g).max()), (pname, idx, fd, an)
            checked += 1
    assert checked >= 6


def test_quantised_mode_is_close_and_on_grid():
    spec = W.tiny_chain(batch=2, size=8, width=8)
    t = W.make_tensors(spec)
    a = evaluate.train_step(spec, t, quant=False)
    b = evaluate.train_step(spec, t, quant=True)
    assert abs(a["loss"] - b["loss"]) < 2e-2 * abs(a["loss"])
    v = b["conv2"].astype(np.float32)
    assert np.all((v.view(np.uint32) & 0xFFFF) == 0)     # bf16-representable
    assert not np.all((a["conv2"].astype(np.float32).view(np.uint32) & 0xFFFF) == 0)


def test_bf16_rounding_nearest_even():
    from workloads import rng
    # 1 + 2^-8 is exactly half way between 1 and 1 + 2^-7: ties go to the even mantissa
    assert rng.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert rng.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert rng.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -12]))[0] == 1.0 + 2.0 ** -7
    x = rng.normal(3, (1000,))
    assert abs(x.mean()) < 0.15 and 0.85 < x.std() < 1.15
    np.testing.assert_array_equal(rng.normal(3, (1000,)), x)
    from oracle.evaluate import _round_bf16
    np.testing.assert_array_equal(_round_bf16(x), rng.round_to_bf16(x))
