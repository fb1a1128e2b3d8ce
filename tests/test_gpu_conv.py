"""Parity of the stand-alone convolution kernels (called through the C ABI) with the fp64 oracle,
element by element, on seeded inputs spanning several tiles and ragged tails.

Tolerance (bf16 outputs): max |gpu - oracle| / max |oracle| <= 1e-2, the bound the workload states;
one bf16 rounding of the result is 2^-9 relative, the fp32 accumulation error is far below that.
Weight gradients are fp32 sums of exact bf16 products: 1e-4."""
import numpy as np
import pytest

import workloads as W
from oracle import ops

pytestmark = pytest.mark.gpu


def dev_bf16(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).cuda()


def dev_f32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def rel_err(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


def make(seed, shape, std=1.0):
    return W.round_to_bf16(W.normal(seed, shape, std))


# (name, n, in_sp, c, k, filt, stride, pad)
CASES = [
    ("cfg1_3x3_c16", 2, (32, 32), 16, 16, (3, 3), 1, 1),
    ("cfg1_first_c3", 2, (32, 32), 3, 16, (3, 3), 1, 1),
    ("1x1_256_64_ragged", 2, (14, 14), 256, 64, (1, 1), 1, 0),
    ("1x1_64_256", 1, (28, 28), 64, 256, (1, 1), 1, 0),
    ("3x3_64_64", 1, (56, 56), 64, 64, (3, 3), 1, 1),
    ("3x3_s2_c32_k64", 3, (15, 15), 32, 64, (3, 3), 2, 1),
    ("1x1_s2", 2, (16, 16), 64, 128, (1, 1), 2, 0),
    ("stem_7x7_s2_c3", 1, (30, 30), 3, 64, (7, 7), 2, 3),
    ("c24_k40", 2, (9, 11), 24, 40, (3, 3), 1, 1),
    ("fc_k10", 2, (1, 1), 16, 10, (1, 1), 1, 0),
    ("head_k4_3d", 1, (4, 5, 6), 32, 4, (1, 1, 1), 1, 0),
    ("3d_3x3x3_c8_k32", 1, (6, 7, 9), 8, 32, (3, 3, 3), 1, 1),
    ("3d_3x3x3_c32_k32", 1, (10, 12, 12), 32, 32, (3, 3, 3), 1, 1),
    ("3d_first_c1", 1, (8, 8, 10), 1, 32, (3, 3, 3), 1, 1),
    ("3d_2x2x2_s2", 1, (8, 8, 8), 16, 24, (2, 2, 2), 2, 0),
    ("big_k_two_ntiles", 1, (12, 12), 128, 256, (3, 3), 1, 1),
    ("1x1_128_128_ragged", 3, (13, 11), 128, 128, (1, 1), 1, 0),
    ("1x1_s2_odd", 2, (15, 17), 128, 64, (1, 1), 2, 0),
    ("1x1_c72_k40", 2, (9, 13), 72, 40, (1, 1), 1, 0),
    ("1x1x1_3d_s2", 1, (6, 7, 9), 64, 64, (1, 1, 1), 2, 0),
    ("3x3_c96_k72", 1, (20, 22), 96, 72, (3, 3), 1, 1),
    ("1x1_320_192", 1, (10, 10), 320, 192, (1, 1), 1, 0),
    # small feature maps: 8 x 8 patches
    ("3x3_7x7_c64_k96", 3, (7, 7), 64, 96, (3, 3), 1, 1),
    ("3x3_9x6_c32_k64", 2, (9, 6), 32, 64, (3, 3), 1, 1),
    # maps at most 7 wide and 8 high with 64 x 64 weight-gradient tiles: two images per patch (odd and even batch)
    ("3x3_5x6_c64_k64_pairs", 4, (5, 6), 64, 64, (3, 3), 1, 1),
    ("3x3_8x7_c128_k64_pairs", 5, (8, 7), 128, 64, (3, 3), 1, 1),
    # first layers with rows longer than one 64-position segment (two segments, the second ragged)
    ("3d_first_c1_wide", 1, (4, 6, 70), 1, 32, (3, 3, 3), 1, 1),
    ("first_c3_wide", 2, (10, 130), 3, 16, (3, 3), 1, 1),
    ("stem_7x7_s2_c3_wide", 2, (20, 200), 3, 64, (7, 7), 2, 3),
    # strided layers with even extents: the data gradient is tiled by residue class (several tiles and a ragged
    # tail per class; a 5x5 window has 3 or 2 taps per class and axis)
    ("3x3_s2_even", 3, (16, 20), 32, 64, (3, 3), 2, 1),
    ("3x3_s2_28_c128", 2, (28, 28), 128, 128, (3, 3), 2, 1),
    ("5x5_s2_even", 2, (12, 16), 16, 24, (5, 5), 2, 2),
    ("3d_3x3x3_s2_even", 1, (8, 6, 10), 16, 32, (3, 3, 3), 2, 1),
    ("1x1_s2_56_c256_k512", 1, (56, 56), 256, 512, (1, 1), 2, 0),
    # enough patches for the resident-filter kernel (several per compute unit), ragged in every axis
    ("rf_3x3_64_64_ragged", 24, (50, 70), 64, 64, (3, 3), 1, 1),
    ("rf_3d_32_32_ragged", 2, (36, 60, 70), 32, 32, (3, 3, 3), 1, 1),
]
IDS = [c[0] for c in CASES]


def tensors(i, n, in_sp, c, k, filt):
    x = make(100 + i, (n,) + in_sp + (c,))
    w = make(200 + i, filt + (c, k), np.sqrt(2.0 / (np.prod(filt) * c)))
    return x, w


@pytest.mark.parametrize("case", CASES, ids=IDS)
@pytest.mark.parametrize("epi", ["plain", "relu", "affine_res_relu", "bias"])
def test_conv_fwd(case, epi):
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad = case
    i = IDS.index(name)
    x, w = tensors(i, n, in_sp, c, k, filt)
    ref = ops.conv_fwd(x, w, stride, pad)
    flags, scale, shift, res = 0, None, None, None
    if epi == "relu":
        flags = A.F_RELU
        ref = ops.relu(ref)
    elif epi == "affine_res_relu":
        flags = A.F_RELU
        scale = 1.0 + 0.1 * W.normal(300 + i, (k,))
        shift = 0.1 * W.normal(400 + i, (k,))
        scale, shift = scale.astype(np.float32).astype(np.float64), shift.astype(np.float32).astype(np.float64)
        res = make(500 + i, ref.shape)
        ref = ops.relu(ops.affine_fwd(ref, scale, shift) + res)
    elif epi == "bias":
        shift = W.normal(600 + i, (k,)).astype(np.float32).astype(np.float64)
        ref = ref + shift
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, flags)
    dx, dw = dev_bf16(x), dev_bf16(w)
    y = torch.full(ref.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(L.conv_workspace_bytes(d, A.CONV_FWD), 256), dtype=torch.uint8, device="cuda")
    ds = dev_f32(scale) if scale is not None else None
    dh = dev_f32(shift) if shift is not None else None
    dr = dev_bf16(res) if res is not None else None
    L.conv_fwd(d, dx.data_ptr(), dw.data_ptr(), ds.data_ptr() if ds is not None else None,
               dh.data_ptr() if dh is not None else None, dr.data_ptr() if dr is not None else None,
               y.data_ptr(), ws.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = host(y)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-2, rel_err(got, ref)
    # element-wise: within one bf16 ulp of the oracle value plus accumulation slack
    assert np.all(np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-3 * np.abs(ref).max())


@pytest.mark.parametrize("case", CASES, ids=IDS)
@pytest.mark.parametrize("epi", ["plain", "addend_mask", "scale"])
def test_conv_dgrad(case, epi):
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad = case
    i = IDS.index(name)
    x, w = tensors(i, n, in_sp, c, k, filt)
    yshape = ops.conv_fwd(x[:1] * 0, w, stride, pad).shape
    dy = make(700 + i, (n,) + yshape[1:])
    scale = addend = mask = None
    weff = w
    if epi == "scale":
        scale = (1.0 + 0.2 * W.normal(800 + i, (k,))).astype(np.float32).astype(np.float64)
        # the kernel rounds w*scale to bf16 before the product
        weff = W.round_to_bf16(w * scale)
    ref = ops.conv_dgrad(dy, weff, x.shape, stride, pad)
    if epi == "addend_mask":
        addend = make(900 + i, x.shape)
        mask = ops.relu(make(1000 + i, x.shape))
        ref = ops.relu_grad(ref + addend, mask)
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
    ddy, dw = dev_bf16(dy), dev_bf16(w)
    out = torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(L.conv_workspace_bytes(d, A.CONV_DGRAD), 256), dtype=torch.uint8, device="cuda")
    ds = dev_f32(scale) if scale is not None else None
    da = dev_bf16(addend) if addend is not None else None
    dm = dev_bf16(mask) if mask is not None else None
    L.conv_dgrad(d, ddy.data_ptr(), dw.data_ptr(), ds.data_ptr() if ds is not None else None,
                 da.data_ptr() if da is not None else None, dm.data_ptr() if dm is not None else None,
                 out.data_ptr(), ws.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = host(out)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-2, rel_err(got, ref)
    if epi == "addend_mask":
        assert np.all(got[mask <= 0] == 0)


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_conv_wgrad(case):
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad = case
    i = IDS.index(name)
    x, w = tensors(i, n, in_sp, c, k, filt)
    yshape = ops.conv_fwd(x[:1] * 0, w, stride, pad).shape
    dy = make(1100 + i, (n,) + yshape[1:])
    ref = ops.conv_wgrad(x, dy, filt, stride, pad)
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
    dxx, ddy = dev_bf16(x), dev_bf16(dy)
    out = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(L.conv_workspace_bytes(d, A.CONV_WGRAD), 256), dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    L.conv_wgrad(d, dxx.data_ptr(), ddy.data_ptr(), out.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-4, rel_err(got, ref)
    # deterministic: a second launch gives the same bits
    out2 = torch.empty_like(out)
    L.conv_wgrad(d, dxx.data_ptr(), ddy.data_ptr(), out2.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_conv_wgrad_bias(case):
    """Weight gradient and bias gradient of a layer in one call: dw has the bits of lms_conv_wgrad, dbias is the
    sum of dy over batch and positions (fp32 sum of exact bf16 values: 1e-4 of the largest sum)."""
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad = case
    i = IDS.index(name)
    x, w = tensors(i, n, in_sp, c, k, filt)
    yshape = ops.conv_fwd(x[:1] * 0, w, stride, pad).shape
    dy = make(1100 + i, (n,) + yshape[1:]) + 0.25          # a non-zero mean: the sums grow with the row count
    dy = W.round_to_bf16(dy)
    ref_b = ops.bias_bwd(dy)
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
    dxx, ddy = dev_bf16(x), dev_bf16(dy)
    dw0 = torch.full((int(np.prod(filt)), c, k), float("nan"), dtype=torch.float32, device="cuda")
    dw1 = torch.full_like(dw0, float("nan"))
    db = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
    need0, need1 = L.conv_workspace_bytes(d, A.CONV_WGRAD), L.conv_workspace_bytes(d, A.CONV_WGRAD_BIAS)
    assert need1 >= need0
    ws = torch.empty(max(need1, 256), dtype=torch.uint8, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    L.conv_wgrad(d, dxx.data_ptr(), ddy.data_ptr(), dw0.data_ptr(), ws.data_ptr(), s)
    L.conv_wgrad_bias(d, dxx.data_ptr(), ddy.data_ptr(), dw1.data_ptr(), db.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    assert torch.equal(dw0, dw1)
    got = db.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert rel_err(got, ref_b) <= 1e-4, rel_err(got, ref_b)
    db2 = torch.full_like(db, float("nan"))
    L.conv_wgrad_bias(d, dxx.data_ptr(), ddy.data_ptr(), dw1.data_ptr(), db2.data_ptr(), ws.data_ptr(), s)
    torch.cuda.synchronize()
    assert torch.equal(db, db2)


def test_empty_and_bad_descriptors_are_rejected():
    import paper_1807_02037_amd as L
    A = L.abi
    with pytest.raises(L.LmsError):
        L.conv_workspace_bytes(L.conv_desc(0, (8, 8), 8, 8, (3, 3), 1, 1), A.CONV_FWD)      # empty batch
    with pytest.raises(L.LmsError):
        L.conv_workspace_bytes(L.conv_desc(1, (2, 2), 8, 8, (5, 5), 1, 0), A.CONV_FWD)      # empty output
    with pytest.raises(L.LmsError):
        L.conv_workspace_bytes(L.conv_desc(1, (8, 8), 8, 8, (3, 3), 0, 1), A.CONV_FWD)      # stride 0


def test_mfma_probe_reports_a_plausible_rate_and_rejects_bad_counts():
    """The matrix-pipe probe (a measurement aid of bench.py): both operand kinds give a rate between a tenth of the
    bf16 peak and the peak, the operation count is the documented one, an iteration count of 0 is LMS_EINVAL."""
    import ctypes
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    fn = A.lib().lms_mfma_probe
    st = torch.cuda.current_stream()
    for rnd in (0, 1):
        flops = ctypes.c_uint64(0)
        assert fn(100, rnd, ctypes.byref(flops), st.cuda_stream) == A.OK
        assert flops.value == 512 * 4 * 100 * 16 * 32768
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        assert fn(5000, rnd, ctypes.byref(flops), st.cuda_stream) == A.OK
        e1.record(st)
        e1.synchronize()
        tflops = flops.value / e0.elapsed_time(e1) / 1e9
        assert 250.0 < tflops < 2600.0, (rnd, tflops)
    assert fn(0, 0, None, st.cuda_stream) == A.EINVAL


RF_CASES = [c for c in CASES if c[0].startswith("rf_")]


@pytest.mark.parametrize("case", RF_CASES, ids=[c[0] for c in RF_CASES])
@pytest.mark.parametrize("terms", ["res_only", "addend_only", "mask_only"])
def test_resident_filter_kernel_single_epilogue_terms(case, terms):
    """The resident-filter kernel is compiled once per combination of epilogue terms (tensor added, ReLU mask,
    per-channel coefficients); the combinations with exactly one tensor term are not reached by the tests above."""
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad = case
    i = IDS.index(name)
    x, w = tensors(i, n, in_sp, c, k, filt)
    s = torch.cuda.current_stream().cuda_stream
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
    if terms == "res_only":
        ref = ops.conv_fwd(x, w, stride, pad)
        res = make(1500 + i, ref.shape)
        ref = ref + res
        y = torch.full(ref.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(max(L.conv_workspace_bytes(d, A.CONV_FWD), 256), dtype=torch.uint8, device="cuda")
        dx, dw, dr = dev_bf16(x), dev_bf16(w), dev_bf16(res)
        L.conv_fwd(d, dx.data_ptr(), dw.data_ptr(), None, None, dr.data_ptr(), y.data_ptr(), ws.data_ptr(), s)
        got = host(y)
    else:
        yshape = ops.conv_fwd(x[:1] * 0, w, stride, pad).shape
        dy = make(1600 + i, (n,) + yshape[1:])
        ref = ops.conv_dgrad(dy, w, x.shape, stride, pad)
        addend = make(1700 + i, x.shape) if terms == "addend_only" else None
        mask = ops.relu(make(1800 + i, x.shape)) if terms == "mask_only" else None
        if addend is not None:
            ref = ref + addend
        if mask is not None:
            ref = ops.relu_grad(ref, mask)
        out = torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(max(L.conv_workspace_bytes(d, A.CONV_DGRAD), 256), dtype=torch.uint8, device="cuda")
        ddy, dw = dev_bf16(dy), dev_bf16(w)
        da = dev_bf16(addend) if addend is not None else None
        dm = dev_bf16(mask) if mask is not None else None
        L.conv_dgrad(d, ddy.data_ptr(), dw.data_ptr(), None, da.data_ptr() if da is not None else None,
                     dm.data_ptr() if dm is not None else None, out.data_ptr(), ws.data_ptr(), s)
        got = host(out)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= 1e-2, rel_err(got, ref)
