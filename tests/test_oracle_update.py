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


def test_momentum_is_the_heavy_ball_recurrence_and_reaches_the_same_minimum():
    """Momentum written without a velocity: p[t+1] - p[t] = mu * (p[t] - p[t-1]) - lr * g[t] (and the plain step for
    t = 0).  Checked on the parameter trajectory the oracle produces, with the gradients recomputed from its
    parameters; mu = 0 is plain gradient descent bit for bit; on the least-squares problem both reach the solution of
    an independent solver, momentum in far fewer steps."""
    spec, tensors = linear_problem()
    lr, mu = 0.3, 0.6
    traj = [dict(tensors)]
    for t in range(1, 6):
        _, params = evaluate.train_steps(spec, tensors, lr, t, momentum=mu)
        traj.append({**tensors, **params})
    for t in range(1, 5):
        g = evaluate.train_step(spec, traj[t])["grad/c.w"]
        lhs = traj[t + 1]["c.w"] - traj[t]["c.w"]
        rhs = mu * (traj[t]["c.w"] - traj[t - 1]["c.w"]) - lr * g
        assert np.allclose(lhs, rhs, rtol=0, atol=1e-13)
    g0 = evaluate.train_step(spec, tensors)["grad/c.w"]
    assert np.allclose(traj[1]["c.w"], tensors["c.w"] - lr * g0, rtol=0, atol=1e-15)
    a = evaluate.train_steps(spec, tensors, lr, 5)
    b = evaluate.train_steps(spec, tensors, lr, 5, momentum=0.0)
    assert a[0] == b[0] and all(np.array_equal(a[1][k], b[1][k]) for k in a[1])
    x = tensors["x"].reshape(-1, 6)
    t_ = tensors["t"].reshape(-1, 3)
    best = np.linalg.lstsq(x, t_, rcond=None)[0]
    _, plain = evaluate.train_steps(spec, tensors, 0.4, 60)
    _, heavy = evaluate.train_steps(spec, tensors, 0.4, 60, momentum=0.5)
    e_plain = np.abs(plain["c.w"].reshape(6, 3) - best).max()
    e_heavy = np.abs(heavy["c.w"].reshape(6, 3) - best).max()
    assert e_heavy < 0.2 * e_plain and e_heavy < 1e-3
