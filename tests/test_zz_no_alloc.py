"""The weight-gradient entry point that allocates nothing (lms_conv_wgrad_static: partial sums in a fixed array of
the library) against lms_conv_wgrad with a caller workspace: bit for bit, on two calls in a row, the second with a
smaller input, and an oversized geometry is refused before anything is launched."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _wgrad_pair(L, n, in_sp, c, k, filt, stride, pad, seed):
    import torch
    A = L.abi
    d = L.conv_desc(n, in_sp, c, k, filt, stride, pad, 0)
    out_sp = tuple((s + 2 * pad - f) // stride + 1 for s, f in zip(in_sp, filt))
    x = torch.from_numpy(W.round_to_bf16(W.normal(seed, (n,) + tuple(in_sp) + (c,))).astype(np.float32)).to(torch.bfloat16).cuda()
    dy = torch.from_numpy(W.round_to_bf16(W.normal(seed + 1, (n,) + out_sp + (k,))).astype(np.float32)).to(torch.bfloat16).cuda()
    stream = torch.cuda.current_stream().cuda_stream
    need = L.conv_workspace_bytes(d, A.CONV_WGRAD)
    assert 0 < need <= L.static_scratch_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = torch.full(tuple(filt) + (c, k), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full_like(ref, float("nan"))
    L.conv_wgrad(d, x.data_ptr(), dy.data_ptr(), ref.data_ptr(), ws.data_ptr(), stream)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    L.conv_wgrad_static(d, x.data_ptr(), dy.data_ptr(), got.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    r, g = ref.cpu().numpy(), got.cpu().numpy()
    assert np.isfinite(r).all()
    assert r.tobytes() == g.tobytes()
    return need


def test_static_wgrad_matches_workspace_wgrad_twice_then_smaller():
    import paper_1807_02037_amd as L
    big = _wgrad_pair(L, 4, (56, 56), 64, 64, (3, 3), 1, 1, seed=7101)          # split partial sums, 3x3
    small = _wgrad_pair(L, 2, (14, 14), 256, 64, (1, 1), 1, 0, seed=7201)       # second call: smaller input, 1x1
    again = _wgrad_pair(L, 1, (10, 12, 12), 32, 32, (3, 3, 3), 1, 1, seed=7301)  # 3-D
    assert big > 0 and small > 0 and again > 0


def test_static_wgrad_refuses_oversized_geometry():
    import torch
    import paper_1807_02037_amd as L
    A = L.abi
    d = L.conv_desc(1, (4, 4, 4), 1024, 1024, (3, 3, 3), 1, 1, 0)    # one partial filter alone is 108 MiB
    assert L.conv_workspace_bytes(d, A.CONV_WGRAD) > L.static_scratch_bytes()
    one = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(L.LmsError, match="fixed scratch"):
        # the size check comes before any pointer is used: nothing is launched
        L.conv_wgrad_static(d, one.data_ptr(), one.data_ptr(), one.data_ptr(), torch.cuda.current_stream().cuda_stream)
