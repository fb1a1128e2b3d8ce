"""Pins of the oracle's update phase: gradient descent on a problem with a known solution, and the first-order
decrease that any correct gradient step must show."""
import numpy as np

import workloads as W
from oracle import evaluate


def linear_problem():
    # one 1x1 convolution without activation and a squared-error loss: a linear least-squares problem in w
    spec = {"name": "linear", "cfg": 9, "ndim": 2, "input": ("x", (4, 5, 5, 6)),
            "layers": [{"name": "c", "op": "conv", "in": "x", "filt": (1, 1), "cout": 3, "stride": 1, "pad": 0,
                        "relu": False, "affine": False, "bias": False, "res": None}],
            "loss": {"op": "mse", "in": "c", "target": "t"}}
    return spec, W.make_tensors(spec)


def test_gradient_descent_converges_to_the_least_squares_solution():
    spec, tensors = linear_problem()
    x = tensors["x"].reshape(-1, 6)
    t = tensors["t"].reshape(-1, 3)
    best = np.linalg.lstsq(x, t, rcond=None)[0]                      # independent library routine
    best_loss = np.mean((x @ best - t) ** 2)
    losses, params = evaluate.train_steps(spec, tensors, lr=0.4, steps=400)
    assert all(b <= a + 1e-15 for a, b in zip(losses, losses[1:]))   # a convex problem with a small step: monotone
    assert np.allclose(params["c.w"].reshape(6, 3), best, atol=1e-6)
    assert abs(losses[-1] - best_loss) < 1e-9


def test_one_small_step_lowers_the_loss_by_lr_times_the_squared_gradient():
    for spec in (W.tiny_chain(), W.pool_net(), W.updown_net()):
        tensors = W.make_tensors(spec, affine="random")
        out = evaluate.train_step(spec, tensors)
        g2 = sum(float((v ** 2).sum()) for k, v in out.items() if k.startswith("grad/"))
        lr = 1e-4 / max(1.0, g2 ** 0.5)
        losses, _ = evaluate.train_steps(spec, tensors, lr, 2)
        assert losses[0] == out["loss"]
        drop = losses[0] - losses[1]
        assert abs(drop - lr * g2) <= 2e-2 * lr * g2, (spec["name"], drop, lr * g2)


def test_quantised_updates_keep_filters_on_the_bf16_grid_only():
    spec = W.tiny_chain()
    tensors = W.make_tensors(spec)
    _, params = evaluate.train_steps(spec, tensors, 1e-2, 2, quant=True)
    for k, v in params.items():
        on_grid = np.array_equal(W.rng.round_to_bf16(v), v)
        assert on_grid == k.endswith(".w"), k
