"""fp32 check mode: the same graphs with fp32 storage and the library's plain fp32 kernels must match the fp64 oracle
(no quantisation anywhere) within 1e-4, loss, forward tensors and every gradient; swapping stays bit-identical."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate

pytestmark = pytest.mark.gpu

SPECS = {
    "tiny_chain": lambda: W.tiny_chain(),
    "pool_net": lambda: W.pool_net(),
    "updown_net": lambda: W.updown_net(),
    "bottleneck_small": lambda: W.bottleneck_stage(batch=2, size=12, cin=32, width=8, blocks=2),
    "resnet_small": lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(1, 1, 1, 1), base=8),
    "unet_small": lambda: W.unet3d(batch=1, size=16, base=8, levels=3),
}


def rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


@pytest.mark.parametrize("name", list(SPECS))
def test_fp32_step_matches_the_exact_oracle(name):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    spec = SPECS[name]()
    tensors = W.make_tensors(spec, affine="random")
    ref = evaluate.train_step(spec, tensors)                 # fp64, nothing rounded
    s = Session(spec, tensors, flags=A.X_KEEP_ALL, dtype=A.F32)
    loss, st = s.step()
    assert abs(loss - ref["loss"]) <= 1e-4 * max(abs(ref["loss"]), 1e-30)
    got = {L_["name"]: s.activation(L_["name"]) for L_ in spec["layers"]}
    got.update(s.grads())
    assert any(k.startswith("grad/") for k in got)
    worst = {}
    for k, v in got.items():
        assert v.shape == ref[k].shape and np.isfinite(v).all(), k
        worst[k] = rel(v, ref[k])
    print(name, "worst:", sorted(worst.items(), key=lambda kv: -kv[1])[:4])
    assert not {k: e for k, e in worst.items() if not e <= 1e-4}
    # the same graph rewritten with swaps: bit-identical in fp32 storage as well
    g0 = s.grad_bits()
    del s
    sw = Session(spec, tensors, rewrite=dict(fuse_swapins=1, lb=2), flags=A.X_POISON | A.X_ENCODE_SWAPS, dtype=A.F32)
    for _ in range(2):
        loss1, st1 = sw.step()
    assert sw.rewrite_stats.tensors_swapped > 0 and st1.bytes_d2h == sw.rewrite_stats.swapped_bytes_out
    assert np.float32(loss1).view(np.uint32) == np.float32(loss).view(np.uint32)
    g1 = sw.grad_bits()
    for k in g0:
        assert np.array_equal(g0[k], g1[k]), k
