"""Update phase on the GPU: several training steps in place, against the oracle's gradient descent."""
import numpy as np
import pytest

import workloads as W
from oracle import evaluate

pytestmark = pytest.mark.gpu

SPECS = {
    "tiny_chain": (lambda: W.tiny_chain(), 0.05),
    "pool_net": (lambda: W.pool_net(), 0.02),
    "updown_net": (lambda: W.updown_net(), 0.02),
    "resnet_small": (lambda: W.resnet50(batch=2, size=32, classes=10, stage_blocks=(1, 1, 1, 1), base=8), 0.02),
}
STEPS = 4


def rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-30)


@pytest.mark.parametrize("name", list(SPECS))
def test_fp32_training_follows_the_oracle(name):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    make, lr = SPECS[name]
    spec = make()
    tensors = W.make_tensors(spec, affine="random")
    ref_losses, ref_params = evaluate.train_steps(spec, tensors, lr, STEPS)
    assert abs(ref_losses[-1] - ref_losses[0]) > 1e-3 * abs(ref_losses[0])      # the steps really move the loss
    s = Session(spec, tensors, dtype=A.F32, lr=lr)
    losses = [s.step()[0] for _ in range(STEPS)]
    print(name, losses, ref_losses)
    for a, b in zip(losses, ref_losses):
        assert abs(a - b) <= 1e-4 * abs(b)
    for k, v in ref_params.items():
        assert rel(s.param(k), v) <= 1e-4, k


@pytest.mark.parametrize("name", ["tiny_chain", "pool_net", "updown_net"])
def test_bf16_training_follows_the_quantised_oracle_and_swapping_changes_nothing(name):
    import paper_1807_02037_amd as L
    from paper_1807_02037_amd.session import Session
    A = L.abi
    make, lr = SPECS[name]
    spec = make()
    tensors = W.make_tensors(spec, affine="random")
    ref_losses, ref_params = evaluate.train_steps(spec, tensors, lr, STEPS, quant=True)
    s = Session(spec, tensors, lr=lr)
    losses = [s.step()[0] for _ in range(STEPS)]
    for a, b in zip(losses, ref_losses):
        assert abs(a - b) <= 1e-2 * abs(b)
    params = {k: s.param(k) for k in ref_params}
    for k, v in ref_params.items():
        assert rel(params[k], v) <= 1e-2, k
    del s
    # the rewritten graph trains bit-identically: swapped tensors, poison fill, encoded copies
    sw = Session(spec, tensors, lr=lr, rewrite=dict(fuse_swapins=1, lb=2), flags=A.X_POISON | A.X_ENCODE_SWAPS)
    assert sw.rewrite_stats.tensors_swapped > 0
    losses_sw = [sw.step()[0] for _ in range(STEPS)]
    assert [np.float32(x).view(np.uint32) for x in losses_sw] == [np.float32(x).view(np.uint32) for x in losses]
    for k in ref_params:
        assert np.array_equal(sw.param(k), params[k]), k
