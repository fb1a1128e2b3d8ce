"""Sampled fp64 checks of convolution-type nodes at sizes where the whole oracle would be too slow:
a few output elements of a node are recomputed one by one from the node's own inputs, straight from
the operation's definition (Section 3.3 only fixes that a backward operation reads forward tensors; the
layer arithmetic is the textbook one, see oracle/ops.py)."""
import itertools

import numpy as np

from paper_1807_02037_amd import abi as A


def _positions(rng, shape, count):
    """Random positions of an (N, spatial...) grid plus its corners (padding paths)."""
    dims = list(shape)
    pos = [tuple(int(rng.integers(0, d)) for d in dims) for _ in range(count)]
    for corner in itertools.product(*[(0, d - 1) for d in dims[1:]]):
        pos.append((int(rng.integers(0, dims[0])),) + corner)
    return pos


def conv_fwd_at(x, w, stride, pad, pos):
    """y[n, o, :] of a cross-correlation with zero padding at one output position."""
    nd = x.ndim - 2
    n, o = pos[0], pos[1:]
    acc = np.zeros(w.shape[-1])
    for tap in np.ndindex(*w.shape[:nd]):
        src = tuple(o[i] * stride + tap[i] - pad for i in range(nd))
        if all(0 <= src[i] < x.shape[1 + i] for i in range(nd)):
            acc += x[(n,) + src] @ w[tap]
    return acc


def conv_dgrad_at(dy, w, stride, pad, pos):
    """dx[n, i, :]: every output position o with o*stride + tap - pad == i contributes dy[n,o,:] @ w[tap]^T."""
    nd = dy.ndim - 2
    n, i = pos[0], pos[1:]
    acc = np.zeros(w.shape[-2])
    for tap in np.ndindex(*w.shape[:nd]):
        t = tuple(i[a] + pad - tap[a] for a in range(nd))
        if any(v < 0 or v % stride for v in t):
            continue
        o = tuple(v // stride for v in t)
        if all(o[a] < dy.shape[1 + a] for a in range(nd)):
            acc += dy[(n,) + o] @ w[tap].T
    return acc


def conv_wgrad_at(x, dy, stride, pad, tap, c, k):
    """dw[tap, c, k] = sum over batch and output positions of x[n, o*stride + tap - pad, c] * dy[n, o, k]."""
    nd = x.ndim - 2
    osp = dy.shape[1:-1]
    xs, ys = [slice(None)], [slice(None)]
    for a in range(nd):
        lo = max(0, -(-(pad - tap[a]) // stride))                       # first o with o*stride + tap - pad >= 0
        hi = min(osp[a] - 1, (x.shape[1 + a] - 1 + pad - tap[a]) // stride)
        if hi < lo:
            return 0.0
        ys.append(slice(lo, hi + 1))
        xs.append(slice(lo * stride + tap[a] - pad, hi * stride + tap[a] - pad + 1, stride))
    return float((x[tuple(xs) + (c,)] * dy[tuple(ys) + (k,)]).sum())


def check_conv_node(rng, info, attr, x, got, samples=40):
    """Compares sampled elements of a convolution-type node with the definition.  x: input arrays in slot
    order (fp64), got: the GPU's output (fp64).  Returns the error relative to the largest |output|."""
    op, f = info.op, attr.flags
    scale_ref = max(np.abs(got).max(), 1e-30)
    worst = 0.0
    if op == A.OP_CONV:
        for pos in _positions(rng, got.shape[:-1], samples):
            y = conv_fwd_at(x[0], x[1], attr.stride, attr.pad, pos)
            i = 2
            if f & A.F_AFFINE:
                y = y * x[i] + x[i + 1]
                i += 2
            if f & A.F_BIAS:
                y = y + x[i]
                i += 1
            if f & A.F_RES:
                y = y + x[i][pos]
            if f & A.F_RELU:
                y = np.maximum(y, 0.0)
            worst = max(worst, np.abs(got[pos] - y).max())
    elif op == A.OP_CONV_DGRAD:
        w, i = x[1], 2
        if f & A.F_AFFINE:
            w = (w * x[i]).astype(np.float32)
            u = w.view(np.uint32).astype(np.uint64)
            w = ((((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16).astype(np.uint32)).view(np.float32).astype(np.float64)
            i += 1
        add = x[i] if f & A.F_ADDEND else None
        i += 1 if f & A.F_ADDEND else 0
        mask = x[i] if f & A.F_MASK else None
        for pos in _positions(rng, got.shape[:-1], samples):
            y = conv_dgrad_at(x[0], w, attr.stride, attr.pad, pos)
            if add is not None:
                y = y + add[pos]
            if mask is not None:
                y = y * (mask[pos] > 0)
            worst = max(worst, np.abs(got[pos] - y).max())
    elif op == A.OP_CONV_WGRAD:
        nd = x[0].ndim - 2
        filt = got.shape[:nd]
        for _ in range(max(8, samples // 3)):
            tap = tuple(int(rng.integers(0, r)) for r in filt)
            c, k = int(rng.integers(0, got.shape[-2])), int(rng.integers(0, got.shape[-1]))
            worst = max(worst, abs(got[tap + (c, k)] - conv_wgrad_at(x[0], x[1], attr.stride, attr.pad, tap, c, k)))
    elif op == A.OP_TCONV:
        for pos in _positions(rng, got.shape[:-1], samples):
            n, o = pos[0], pos[1:]
            src = tuple(v // 2 for v in o)
            tap = tuple(v % 2 for v in o)
            worst = max(worst, np.abs(got[pos] - x[0][(n,) + src] @ x[1][tap]).max())
    elif op == A.OP_TCONV_DGRAD:
        nd = got.ndim - 2
        add = x[2] if f & A.F_ADDEND else None
        mask = x[2 + (1 if f & A.F_ADDEND else 0)] if f & A.F_MASK else None
        for pos in _positions(rng, got.shape[:-1], samples):
            n, d = pos[0], pos[1:]
            y = np.zeros(got.shape[-1])
            for tap in np.ndindex(*(2,) * nd):
                y += x[0][(n,) + tuple(2 * d[a] + tap[a] for a in range(nd))] @ x[1][tap].T
            if add is not None:
                y = y + add[pos]
            if mask is not None:
                y = y * (mask[pos] > 0)
            worst = max(worst, np.abs(got[pos] - y).max())
    elif op == A.OP_TCONV_WGRAD:
        nd = x[0].ndim - 2
        for _ in range(max(8, samples // 3)):
            tap = tuple(int(rng.integers(0, 2)) for _ in range(nd))
            c, k = int(rng.integers(0, got.shape[-2])), int(rng.integers(0, got.shape[-1]))
            sl = (slice(None),) + tuple(slice(t, None, 2) for t in tap)
            ref = float((x[0][..., c] * x[1][sl + (k,)]).sum())
            worst = max(worst, abs(got[tap + (c, k)] - ref))
    else:
        raise ValueError(op)
    return worst / scale_ref


CONV_OPS = (A.OP_CONV, A.OP_CONV_DGRAD, A.OP_CONV_WGRAD, A.OP_TCONV, A.OP_TCONV_DGRAD, A.OP_TCONV_WGRAD)
