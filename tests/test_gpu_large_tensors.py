"""Stand-alone convolution entry points on activations of 2 GiB and more, against the sampled fp64 oracle.

Above 2 GiB the kernels leave their 32-bit buffer-offset paths (the resident-filter 3x3 kernel and the patch weight
gradient fall back, the first-layer gather is per image) and every row index needs 64-bit arithmetic; ResNet-50 at
the batches a 16 GB cap allows with swapping produces such tensors (6 GB at batch 3772).  Inputs are seeded N(0,1)
draws made on the device; forward / data-gradient outputs are compared on >= 4096 sampled elements including the last
rows of the tensor, weight gradients on whole filter taps summed over every position."""
from types import SimpleNamespace

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

GIB2 = 1 << 31

# name, n, in_sp, c, k, filt, stride, pad, passes
CASES = [
    ("pw_64_256", 1400, (56, 56), 64, 256, (1, 1), 1, 0, ("fwd", "dgrad", "wgrad")),
    ("pw_256_64", 1400, (56, 56), 256, 64, (1, 1), 1, 0, ("fwd", "dgrad", "wgrad")),
    ("3x3_64_64", 5400, (56, 56), 64, 64, (3, 3), 1, 1, ("fwd", "dgrad", "wgrad")),
    ("stem_7x7_s2", 1400, (224, 224), 3, 64, (7, 7), 2, 3, ("fwd", "wgrad")),
    ("3d_32_32", 5, (192, 192, 192), 32, 32, (3, 3, 3), 1, 1, ("fwd", "dgrad", "wgrad")),
    ("1x1_s2_256_512", 1400, (56, 56), 256, 512, (1, 1), 2, 0, ("fwd", "dgrad", "wgrad")),
]


def _rand(gen, shape, std=1.0):
    import torch
    t = torch.empty(shape, device="cuda", dtype=torch.bfloat16)
    t.normal_(0.0, std, generator=gen)
    return t


def _tail_positions(shape, channels):
    """The last positions of the tensor (largest byte offsets) as extra samples."""
    n = shape[0]
    return np.asarray([[n - 1] + [d - 1 - (i % d) for d in shape[1:]] for i in range(8)], dtype=np.int64)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_entry_points_on_tensors_of_2gib_and_more(case):
    import torch
    import paper_1807_02037_amd as L
    import sampled_oracle as S
    A = L.abi
    name, n, in_sp, c, k, filt, stride, pad, passes = case
    out_sp = tuple((s + 2 * pad - f) // stride + 1 for s, f in zip(in_sp, filt))
    xs, ys = (n,) + in_sp + (c,), (n,) + out_sp + (k,)
    assert max(int(np.prod(xs)), int(np.prod(ys))) * 2 >= GIB2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1807020370 + len(name))
    rng = np.random.default_rng(len(name))
    stream = torch.cuda.current_stream().cuda_stream
    fan_in = c * int(np.prod(filt))
    w = _rand(gen, tuple(filt) + (c, k), (2.0 / fan_in) ** 0.5)
    attr = SimpleNamespace(flags=0, stride=stride, pad=pad)

    def ws_for(d, which):
        return torch.empty(max(L.conv_workspace_bytes(d, which), 256), dtype=torch.uint8, device="cuda")
    if "fwd" in passes:
        print(name, "fwd", flush=True)
        d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, A.F_RELU)
        x, res = _rand(gen, xs), _rand(gen, ys)
        scale = (1.0 + 0.1 * torch.randn(k, device="cuda", generator=gen)).float()
        shift = (0.1 * torch.randn(k, device="cuda", generator=gen)).float()
        y = torch.empty(ys, device="cuda", dtype=torch.bfloat16)
        ws = ws_for(d, A.CONV_FWD)
        L.conv_fwd(d, x.data_ptr(), w.data_ptr(), scale.data_ptr(), shift.data_ptr(), res.data_ptr(), y.data_ptr(), ws.data_ptr(), stream)
        torch.cuda.synchronize()
        attr.flags = A.F_AFFINE | A.F_RES | A.F_RELU
        e, cnt = S.check_conv_node(rng, SimpleNamespace(op=A.OP_CONV), attr, [x, w, scale, shift, res], y, samples=64)
        assert cnt >= S.MIN_ELEMENTS and e <= 1e-2, (name, "fwd", e)
        tail = _tail_positions(ys[:-1], k)
        ref = np.maximum(S.conv_fwd_at(x, w, stride, pad, tail) * S._host(scale) + S._host(shift) + S._take(res, list(tail.T)), 0.0)
        assert np.abs(S._take(y, list(tail.T)) - ref).max() <= 1e-2 * float(y.abs().max()), (name, "fwd tail")
        del x, res, y, ws
        torch.cuda.empty_cache()
    if "dgrad" in passes:
        print(name, "dgrad", flush=True)
        d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
        dy, add, mask = _rand(gen, ys), _rand(gen, xs), _rand(gen, xs)
        dx = torch.empty(xs, device="cuda", dtype=torch.bfloat16)
        ws = ws_for(d, A.CONV_DGRAD)
        L.conv_dgrad(d, dy.data_ptr(), w.data_ptr(), None, add.data_ptr(), mask.data_ptr(), dx.data_ptr(), ws.data_ptr(), stream)
        torch.cuda.synchronize()
        attr.flags = A.F_ADDEND | A.F_MASK
        e, cnt = S.check_conv_node(rng, SimpleNamespace(op=A.OP_CONV_DGRAD), attr, [dy, w, add, mask], dx, samples=64)
        assert cnt >= S.MIN_ELEMENTS and e <= 1e-2, (name, "dgrad", e)
        tail = _tail_positions(xs[:-1], c)
        ref = (S.conv_dgrad_at(dy, w, stride, pad, tail) + S._take(add, list(tail.T))) * (S._take(mask, list(tail.T)) > 0)
        assert np.abs(S._take(dx, list(tail.T)) - ref).max() <= 1e-2 * float(dx.abs().max()), (name, "dgrad tail")
        del dy, add, mask, dx, ws
        torch.cuda.empty_cache()
    if "wgrad" in passes:
        print(name, "wgrad", flush=True)
        d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
        x, dy = _rand(gen, xs), _rand(gen, ys)
        dw = torch.full(tuple(filt) + (c, k), float("nan"), device="cuda", dtype=torch.float32)
        ws = ws_for(d, A.CONV_WGRAD)
        L.conv_wgrad(d, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), ws.data_ptr(), stream)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(dw).all())
        attr.flags = 0
        # two taps (both padding sides) are enough above 2 GiB: every tap sums over the whole tensor
        taps = S.sample_taps(rng, tuple(filt), c, k)[:2]
        got = dw.double().cpu().numpy()
        scale_ref = np.abs(got).max()
        for tap in taps:
            ref = S.conv_wgrad_tap(x, dy, stride, pad, tap)
            assert np.abs(got[tap] - ref).max() <= 1e-4 * scale_ref, (name, "wgrad", tap)
