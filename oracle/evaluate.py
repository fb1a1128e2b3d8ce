"""Runs a graph vertex by vertex in topological order, in fp64.

TEST INFRASTRUCTURE ONLY; nothing in the product path may import it.

An operation runs once all its incoming edges carry data (Section 3.2); swap-out
and swap-in vertices are identity functions (Eq. 2, Eq. 5), so a rewritten graph
must produce bit-identical values.  With quant=True every tensor the GPU path
stores in bfloat16 (vertices marked "q") is rounded to bfloat16 (nearest even)
right after it is computed, all arithmetic staying in fp64.
"""
import numpy as np

from . import ops


def _round_bf16(a):
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def run(g, feeds, quant=False, order=None):
    """feeds: {variable name: array}.  Returns {vertex id: value}."""
    gam = g.gamma()
    if order is None:
        order = sorted((n.id for n in g.nodes), key=lambda v: (gam[v], v))
    val = {}
    for v in order:
        n = g.nodes[v]
        if n.is_var:
            a = feeds[n.name]
            val[v] = a if a.dtype.kind == "i" else np.asarray(a, dtype=np.float64)
            continue
        x = [val[i] for i in g.inputs(v)]
        a = n.attrs
        k = n.op
        if k in ("swap_out", "swap_in", "identity"):
            r = x[0]
        elif k == "conv":
            r = ops.conv_fwd(x[0], x[1], a["stride"], a["pad"])
        elif k == "affine":
            r = ops.affine_fwd(x[0], x[1], x[2])
        elif k == "bias":
            r = x[0] + x[1]
        elif k == "add":
            r = x[0] + x[1]
        elif k == "relu":
            r = ops.relu(x[0])
        elif k == "maxpool":
            r = ops.maxpool_fwd(x[0], a["win"], a["stride"], a["pad"])[0]
        elif k == "gap":
            r = ops.gap_fwd(x[0])
        elif k == "tconv":
            r = ops.tconv_fwd(x[0], x[1])
        elif k == "concat":
            r = ops.concat(x[0], x[1])
        elif k == "mse":
            r = np.float64(ops.mse_fwd(x[0], x[1]))
        elif k == "softmax_ce":
            r = np.float64(ops.softmax_ce_fwd(x[0], x[1]))
        elif k == "mse_bwd":
            r = ops.mse_bwd(x[0], x[1])
        elif k == "softmax_ce_bwd":
            r = ops.softmax_ce_bwd(x[0], x[1])
        elif k == "relu_grad":
            r = ops.relu_grad(x[0], x[1])
        elif k == "bias_grad":
            r = ops.bias_bwd(x[0])
        elif k == "affine_dscale":
            r = ops.affine_bwd(x[0], x[1], 1.0)[1]
        elif k == "affine_dx":
            r = x[0] * x[1]
        elif k == "conv_wgrad":
            filt = val[a["filt_of"]].shape[:-2]
            r = ops.conv_wgrad(x[0], x[1], filt, a["stride"], a["pad"])
        elif k == "conv_dgrad":
            r = ops.conv_dgrad(x[0], x[1], val[a["shape_of"]].shape, a["stride"], a["pad"])
        elif k == "tconv_wgrad":
            r = ops.tconv_wgrad(x[0], x[1])
        elif k == "tconv_dgrad":
            r = ops.tconv_dgrad(x[0], x[1])
        elif k == "maxpool_bwd":
            arg = ops.maxpool_fwd(x[1], a["win"], a["stride"], a["pad"])[1]
            r = ops.maxpool_bwd(x[0], arg, x[1].shape, a["win"], a["stride"], a["pad"])
        elif k == "gap_bwd":
            r = ops.gap_bwd(x[0], val[a["shape_of"]].shape)
        elif k == "slice_c":
            ca = val[a["shape_of"]].shape[-1]
            r = ops.concat_bwd(x[0], ca)[1 if a["second"] else 0]
        else:
            raise ValueError(k)
        if quant and a.get("q") and isinstance(r, np.ndarray) and r.ndim > 0:
            r = _round_bf16(r)
        val[v] = r
    return val


def train_step(spec, tensors, quant=False):
    """Loss, parameter gradients and layer outputs of one forward+backward pass of a workload.
    Returns {"loss": float, "grad/<param>": array, "<layer>": array}."""
    from . import model
    g, ids = model.build(spec)
    val = run(g, tensors, quant)
    return {name: val[v] for name, v in ids.items() if not g.nodes[v].is_var}


def train_steps(spec, tensors, lr, steps, quant=False, momentum=0.0):
    """Update phase (Section 3.3: after the backward phase every learnable parameter p takes an update computed from
    its gradient; the same batch every step).  Plain gradient descent, p <- p - lr * dL/dp, or with momentum > 0 the
    classical momentum rule: v <- momentum * v + dL/dp (v starts at zero), p <- p - lr * v.  Returns
    (losses per step, parameters after the last step).  With quant the filters, which the GPU stores in bf16,
    are rounded to bf16 after each update; per-channel scale / shift / bias and the velocities stay unrounded
    (fp32 on the GPU)."""
    cur = dict(tensors)
    vel = {}
    losses = []
    for _ in range(steps):
        out = train_step(spec, cur, quant)
        losses.append(float(out["loss"]))
        for name, g in out.items():
            if not name.startswith("grad/"):
                continue
            p = name[len("grad/"):]
            if momentum:
                vel[p] = momentum * vel.get(p, 0.0) + g
                step = vel[p]
            else:
                step = g
            new = cur[p] - lr * step
            if quant and p.endswith(".w"):
                new = _round_bf16(new)
            cur[p] = new
    return losses, {k: v for k, v in cur.items() if "grad/" + k in out}
