"""Parity of the convolution entry points with the fp64 oracle on seeded random geometries.

The named cases of test_gpu_conv.py pick shapes for particular kernels; here the geometry is drawn (seeded), so the
routing between the kernels (which depends on channel counts, window, stride, padding and extents) is exercised on
combinations nobody chose by hand.  Every drawn geometry is valid (non-empty output); tolerances as in
test_gpu_conv.py."""
import numpy as np
import pytest

import workloads as W
from oracle import ops

pytestmark = pytest.mark.gpu

CHANNELS = [1, 3, 4, 8, 16, 24, 32, 40, 64, 72, 96, 128]


def draw_case(seed):
    r = np.random.RandomState(seed)
    nd = 2 if r.rand() < 0.65 else 3
    f = int(r.choice([1, 2, 3, 5, 7] if nd == 2 else [1, 2, 3]))
    stride = int(r.choice([1, 2]))
    pad = int(r.randint(0, f // 2 + 1))
    c = int(r.choice(CHANNELS))
    k = int(r.choice([4, 8, 10, 16, 24, 32, 40, 64, 96, 128]))
    hi = 40 if nd == 2 else 14
    sp = tuple(int(r.randint(max(f, 2), hi + 1)) for _ in range(nd))
    if r.rand() < 0.3:          # one long axis: rows of more than one 64-position segment
        sp = sp[:-1] + (int(r.randint(64, 150)),)
    if stride == 2 and r.rand() < 0.6:          # even extents: the strided data gradient tiles by residue class
        sp = tuple(v + (v & 1) for v in sp)
    n = int(r.randint(1, 4))
    # keep the oracle's work to a second or so
    while n * np.prod(sp) * c * k * f ** nd > 6e9:
        sp = tuple(max(f, s // 2) for s in sp)
    return n, sp, c, k, (f,) * nd, stride, pad


SEEDS = list(range(80))


def dev_bf16(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()


def rel_err(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


def make(seed, shape, std=1.0):
    return W.round_to_bf16(W.normal(seed, shape, std))


@pytest.mark.parametrize("seed", SEEDS)
def test_random_geometry_fwd_dgrad_wgrad(seed):
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    n, sp, c, k, filt, stride, pad = draw_case(seed)
    print("case", seed, n, sp, c, k, filt, stride, pad, flush=True)
    x = make(5000 + seed, (n,) + sp + (c,))
    w = make(6000 + seed, filt + (c, k), np.sqrt(2.0 / (np.prod(filt) * c)))
    y_ref = ops.conv_fwd(x, w, stride, pad)
    dy = make(7000 + seed, y_ref.shape)
    s = torch.cuda.current_stream().cuda_stream
    d = L.conv_desc(n, sp, c, k, filt, stride, pad, A.F_RELU)
    wsb = max(L.conv_workspace_bytes(d, which) for which in (A.CONV_FWD, A.CONV_DGRAD, A.CONV_WGRAD))
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    dx_, dw_, ddy = dev_bf16(x), dev_bf16(w), dev_bf16(dy)

    y = torch.full(y_ref.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    if seed % 2 == 0:
        L.conv_fwd(d, dx_.data_ptr(), dw_.data_ptr(), None, None, None, y.data_ptr(), ws.data_ptr(), s)
        ref = ops.relu(y_ref)
    else:                                        # per-channel scale and shift, residual, ReLU
        scale = (1.0 + 0.2 * W.normal(8000 + seed, (k,))).astype(np.float32)
        shift = (0.1 * W.normal(8100 + seed, (k,))).astype(np.float32)
        res = make(8200 + seed, y_ref.shape)
        ds, dh, dr = torch.from_numpy(scale).cuda(), torch.from_numpy(shift).cuda(), dev_bf16(res)
        L.conv_fwd(d, dx_.data_ptr(), dw_.data_ptr(), ds.data_ptr(), dh.data_ptr(), dr.data_ptr(), y.data_ptr(), ws.data_ptr(), s)
        ref = ops.relu(y_ref * scale.astype(np.float64) + shift.astype(np.float64) + res)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-2

    d0 = L.conv_desc(n, sp, c, k, filt, stride, pad, 0)
    dx = torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ref = ops.conv_dgrad(dy, w, x.shape, stride, pad)
    if seed % 3 == 0:                            # gradient accumulation and the ReLU mask of the producer
        addend = make(8300 + seed, x.shape)
        mask = ops.relu(make(8400 + seed, x.shape))
        da, dm = dev_bf16(addend), dev_bf16(mask)
        L.conv_dgrad(d0, ddy.data_ptr(), dw_.data_ptr(), None, da.data_ptr(), dm.data_ptr(), dx.data_ptr(), ws.data_ptr(), s)
        ref = ops.relu_grad(ref + addend, mask)
    else:
        L.conv_dgrad(d0, ddy.data_ptr(), dw_.data_ptr(), None, None, None, dx.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    got = dx.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-2

    dw = torch.full(w.shape, float("nan"), dtype=torch.float32, device="cuda")
    L.conv_wgrad(d0, dx_.data_ptr(), ddy.data_ptr(), dw.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    got = dw.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_err(got, ops.conv_wgrad(x, dy, filt, stride, pad)) <= 1e-4
