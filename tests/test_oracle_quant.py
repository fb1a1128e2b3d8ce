"""Why the bf16 parity gate compares with the oracle run with bf16 storage points, shown with the oracle alone.

ReLU masks are binary decisions on stored values.  Rounding one forward activation to bf16 (at most 2^-8 of an element)
changes which elements of the next layers are positive, and that alone moves a weight gradient by more than the
1e-2 the workload allows, with every other operation exact in fp64.  So a GPU path that stores activations in bf16
cannot be held to 1e-2 against an oracle that never rounds, whatever its arithmetic; it can be held to it against
the same fp64 arithmetic with the roundings where the stored tensors are.  Where exactly the backward roundings sit
(a gradient rounded before or after it is added to another one) changes gradients by far less than the bound."""
import numpy as np

import workloads as W
from quant_marks import run_with_marks


def rel(a, b):
    return np.abs(a - b).max() / np.abs(b).max()


def grads(d):
    return {k: v for k, v in d.items() if k.startswith("grad/")}


def test_one_forward_rounding_moves_a_weight_gradient_by_a_percent():
    spec = W.tiny_chain()
    t = W.make_tensors(spec, affine="random")
    exact = run_with_marks(spec, t, "none")
    one = run_with_marks(spec, t, {"conv1"})
    # the rounded tensor itself moves by at most half a bf16 step, the loss hardly at all
    assert rel(one["conv1"], exact["conv1"]) <= 2.0 ** -8
    assert abs(one["loss"] - exact["loss"]) <= 1e-3 * abs(exact["loss"])
    moved = {k: rel(one[k], exact[k]) for k in grads(exact)}
    worst = max(moved, key=moved.get)
    assert worst == "grad/conv2.w" and 8e-3 <= moved[worst] <= 1.5e-2, moved
    # the mechanism: ReLU decisions downstream of the rounded tensor flip, nothing upstream changes
    flips = sum(int(((one[n] > 0) != (exact[n] > 0)).sum()) for n in ("conv2", "conv3", "conv4"))
    assert flips > 0 and not ((one["conv1"] > 0) != (exact["conv1"] > 0)).any()


def test_full_storage_rounding_moves_gradients_beyond_the_bound_on_both_small_configs():
    for spec, lo, hi in ((W.tiny_chain(), 5e-3, 2e-2),
                         (W.bottleneck_stage(batch=2, size=14, cin=64, width=16, blocks=3), 1e-2, 8e-2)):
        t = W.make_tensors(spec, affine="random")
        exact = run_with_marks(spec, t, "none")
        quant = run_with_marks(spec, t, "model")
        worst = max(rel(quant[k], exact[k]) for k in grads(exact))
        assert lo <= worst <= hi, (spec["name"], worst)
        # loss and forward tensors stay inside 1e-2
        assert abs(quant["loss"] - exact["loss"]) <= 1e-2 * abs(exact["loss"])
        for L in spec["layers"]:
            assert rel(quant[L["name"]], exact[L["name"]]) <= 1e-2, L["name"]


def test_placement_of_backward_roundings_changes_gradients_far_less_than_the_bound():
    for spec in (W.tiny_chain(), W.bottleneck_stage(batch=2, size=14, cin=64, width=16, blocks=3), W.pool_net(),
                 W.updown_net()):
        t = W.make_tensors(spec, affine="random")
        a = run_with_marks(spec, t, "model")
        b = run_with_marks(spec, t, "all_backward")
        assert a["loss"] == b["loss"]
        for L in spec["layers"]:
            assert np.array_equal(a[L["name"]], b[L["name"]])        # forward pass untouched
        for k in grads(a):
            assert rel(b[k], a[k]) <= 5e-3, (spec["name"], k, rel(b[k], a[k]))


def test_forward_marks_are_exactly_the_layer_outputs():
    """The forward storage points are the outputs of the library's operations (one tensor per layer: convolution
    with its affine / residual / ReLU applied, pooling, concatenation), not a choice made per kernel."""
    from oracle import model
    from oracle.graph import FWD
    for spec in (W.tiny_chain(), W.pool_net(), W.updown_net(), W.resnet50(batch=1, size=32)):
        g, ids = model.build(spec)
        layer_ids = {ids[L["name"]] for L in spec["layers"]}
        marked = {n.id for n in g.nodes if not n.is_var and n.phase == FWD and n.attrs.get("q")}
        assert marked == layer_ids
