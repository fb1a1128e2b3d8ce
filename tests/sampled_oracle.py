"""Sampled fp64 checks of convolution-type nodes at sizes where the whole oracle would be too slow:
at least 4096 output elements of a node are recomputed from the node's own inputs, straight from the
operation's definition (Section 3.3 only fixes that a backward operation reads forward tensors; the
layer arithmetic is the textbook one, see oracle/ops.py).  Forward and data-gradient nodes are sampled by
output position (all channels of a position), weight gradients by filter tap (the whole channel x channel
slice of a tap, summed over every position of the layer).

Inputs may be fp64 numpy arrays or device tensors (torch, bf16 / fp32): only the sampled rows, or one batch
chunk at a time, are brought to the host, so tensors of several GiB can be checked."""
import itertools

import numpy as np

from paper_1807_02037_amd import abi as A

MIN_ELEMENTS = 4096


def _is_torch(t):
    return type(t).__module__.startswith("torch")


def _take(t, idx):
    """t[idx] (advanced indexing over the leading axes) as an fp64 numpy array."""
    if _is_torch(t):
        import torch
        dev = [torch.as_tensor(np.ascontiguousarray(i), device=t.device) for i in idx]
        return t[tuple(dev)].double().cpu().numpy()
    return np.asarray(t[tuple(idx)], dtype=np.float64)


def _host(t):
    """A whole (small) tensor as fp64 numpy."""
    if _is_torch(t):
        return t.double().cpu().numpy()
    return np.asarray(t, dtype=np.float64)


def _chunk(t, lo, hi):
    """t[lo:hi] along the batch axis as fp64 numpy."""
    if _is_torch(t):
        return t[lo:hi].double().cpu().numpy()
    return np.asarray(t[lo:hi], dtype=np.float64)


def sample_positions(rng, shape, count):
    """`count` random positions of an (N, spatial...) grid plus all its corners (padding paths): int array
    (S, 1 + nd)."""
    dims = list(shape)
    pos = [[int(rng.integers(0, d)) for d in dims] for _ in range(count)]
    for corner in itertools.product(*[sorted({0, d - 1}) for d in dims[1:]]):
        pos.append([int(rng.integers(0, dims[0]))] + list(corner))
    return np.asarray(pos, dtype=np.int64)


def conv_fwd_at(x, w, stride, pad, pos):
    """y[n, o, :] of a cross-correlation with zero padding at the output positions pos (S, 1+nd): (S, K)."""
    nd = pos.shape[1] - 1
    w = _host(w)
    acc = np.zeros((pos.shape[0], w.shape[-1]))
    for tap in np.ndindex(*w.shape[:nd]):
        src = [pos[:, 1 + a] * stride + tap[a] - pad for a in range(nd)]
        ok = np.ones(pos.shape[0], dtype=bool)
        for a in range(nd):
            ok &= (src[a] >= 0) & (src[a] < x.shape[1 + a])
        if not ok.any():
            continue
        rows = _take(x, [pos[ok, 0]] + [s[ok] for s in src])
        acc[ok] += rows @ w[tap]
    return acc


def conv_dgrad_at(dy, w, stride, pad, pos):
    """dx[n, i, :]: every output position o with o*stride + tap - pad == i contributes dy[n,o,:] @ w[tap]^T."""
    nd = pos.shape[1] - 1
    w = _host(w)
    acc = np.zeros((pos.shape[0], w.shape[-2]))
    for tap in np.ndindex(*w.shape[:nd]):
        t = [pos[:, 1 + a] + pad - tap[a] for a in range(nd)]
        ok = np.ones(pos.shape[0], dtype=bool)
        for a in range(nd):
            ok &= (t[a] >= 0) & (t[a] % stride == 0) & (t[a] // stride < dy.shape[1 + a])
        if not ok.any():
            continue
        rows = _take(dy, [pos[ok, 0]] + [v[ok] // stride for v in t])
        acc[ok] += rows @ w[tap].T
    return acc


def conv_wgrad_tap(x, dy, stride, pad, tap, batch_chunk=None):
    """dw[tap, :, :] = sum over batch and output positions of x[n, o*stride + tap - pad, :] (x) dy[n, o, :]: (C, K)."""
    nd = len(tap)
    osp = dy.shape[1:-1]
    xs, ys = [], []
    for a in range(nd):
        lo = max(0, -(-(pad - tap[a]) // stride))                       # first o with o*stride + tap - pad >= 0
        hi = min(osp[a] - 1, (x.shape[1 + a] - 1 + pad - tap[a]) // stride)
        if hi < lo:
            return np.zeros((x.shape[-1], dy.shape[-1]))
        ys.append(slice(lo, hi + 1))
        xs.append(slice(lo * stride + tap[a] - pad, hi * stride + tap[a] - pad + 1, stride))
    n = x.shape[0]
    if batch_chunk is None:
        per = int(np.prod(x.shape[1:])) + int(np.prod(dy.shape[1:]))
        batch_chunk = max(1, (1 << 27) // max(per, 1))                  # about 1 GiB of fp64 per chunk
    out = np.zeros((x.shape[-1], dy.shape[-1]))
    for lo in range(0, n, batch_chunk):
        hi = min(n, lo + batch_chunk)
        xa = _chunk(x, lo, hi)[(slice(None),) + tuple(xs)]
        ya = _chunk(dy, lo, hi)[(slice(None),) + tuple(ys)]
        out += xa.reshape(-1, xa.shape[-1]).T @ ya.reshape(-1, ya.shape[-1])
    return out


def sample_taps(rng, filt, c, k):
    """Filter taps whose (c, k) slices together hold at least MIN_ELEMENTS entries: the first and the last tap
    (both padding sides) and random ones."""
    all_taps = list(np.ndindex(*filt))
    want = min(len(all_taps), max(2, -(-MIN_ELEMENTS // (c * k))))
    taps = [all_taps[0], all_taps[-1]] if len(all_taps) > 1 else [all_taps[0]]
    rest = [t for t in all_taps if t not in taps]
    order = rng.permutation(len(rest))
    for i in order[:max(0, want - len(taps))]:
        taps.append(rest[int(i)])
    return taps[:max(want, 1)]


def n_positions(samples, channels):
    return max(samples, -(-MIN_ELEMENTS // channels))


def check_conv_node(rng, info, attr, x, got, samples=40):
    """Compares sampled elements of a convolution-type node with the definition.  x: inputs in slot order, got:
    the GPU's output (fp64 arrays or device tensors).  Returns (error relative to the largest |output|, number of
    output elements compared)."""
    op, f = info.op, attr.flags
    gshape = tuple(got.shape)
    scale_ref = float(got.abs().max()) if _is_torch(got) else float(np.abs(got).max())
    scale_ref = max(scale_ref, 1e-30)
    worst, count = 0.0, 0

    def at(t, pos):
        return _take(t, [pos[:, i] for i in range(pos.shape[1])])

    if op == A.OP_CONV:
        pos = sample_positions(rng, gshape[:-1], n_positions(samples, gshape[-1]))
        y = conv_fwd_at(x[0], x[1], attr.stride, attr.pad, pos)
        i = 2
        if f & A.F_AFFINE:
            y = y * _host(x[i]) + _host(x[i + 1])
            i += 2
        if f & A.F_BIAS:
            y = y + _host(x[i])
            i += 1
        if f & A.F_RES:
            y = y + at(x[i], pos)
        if f & A.F_RELU:
            y = np.maximum(y, 0.0)
        worst, count = np.abs(at(got, pos) - y).max(), y.size
    elif op == A.OP_CONV_DGRAD:
        w, i = _host(x[1]), 2
        if f & A.F_AFFINE:
            w = (w * _host(x[i])).astype(np.float32)
            u = w.view(np.uint32).astype(np.uint64)
            w = ((((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16).astype(np.uint32)).view(np.float32).astype(np.float64)
            i += 1
        add = x[i] if f & A.F_ADDEND else None
        i += 1 if f & A.F_ADDEND else 0
        mask = x[i] if f & A.F_MASK else None
        pos = sample_positions(rng, gshape[:-1], n_positions(samples, gshape[-1]))
        y = conv_dgrad_at(x[0], w, attr.stride, attr.pad, pos)
        if add is not None:
            y = y + at(add, pos)
        if mask is not None:
            y = y * (at(mask, pos) > 0)
        worst, count = np.abs(at(got, pos) - y).max(), y.size
    elif op == A.OP_CONV_WGRAD:
        nd = len(x[0].shape) - 2
        for tap in sample_taps(rng, gshape[:nd], gshape[-2], gshape[-1]):
            ref = conv_wgrad_tap(x[0], x[1], attr.stride, attr.pad, tap)
            g = _chunk(got, tap[0], tap[0] + 1)[0][tuple(tap[1:])]
            worst = max(worst, np.abs(g - ref).max())
            count += ref.size
    elif op == A.OP_TCONV:
        pos = sample_positions(rng, gshape[:-1], n_positions(samples, gshape[-1]))
        src = np.concatenate([pos[:, :1], pos[:, 1:] // 2], axis=1)
        rows = at(x[0], src)
        w = _host(x[1])
        y = np.einsum("sc,sck->sk", rows, w[tuple((pos[:, 1:] % 2).T)])
        worst, count = np.abs(at(got, pos) - y).max(), y.size
    elif op == A.OP_TCONV_DGRAD:
        nd = len(gshape) - 2
        add = x[2] if f & A.F_ADDEND else None
        mask = x[2 + (1 if f & A.F_ADDEND else 0)] if f & A.F_MASK else None
        pos = sample_positions(rng, gshape[:-1], n_positions(samples, gshape[-1]))
        w = _host(x[1])
        y = np.zeros((pos.shape[0], gshape[-1]))
        for tap in np.ndindex(*(2,) * nd):
            src = np.concatenate([pos[:, :1], 2 * pos[:, 1:] + np.asarray(tap)], axis=1)
            y += at(x[0], src) @ w[tap].T
        if add is not None:
            y = y + at(add, pos)
        if mask is not None:
            y = y * (at(mask, pos) > 0)
        worst, count = np.abs(at(got, pos) - y).max(), y.size
    elif op == A.OP_TCONV_WGRAD:
        nd = len(x[0].shape) - 2
        for tap in sample_taps(rng, (2,) * nd, gshape[-2], gshape[-1]):
            # window = stride = 2 without padding: the adjoint of a stride-2 convolution from the large grid
            ref = conv_wgrad_tap(x[1], x[0], 2, 0, tap).T
            g = _chunk(got, tap[0], tap[0] + 1)[0][tuple(tap[1:])]
            worst = max(worst, np.abs(g - ref).max())
            count += ref.size
    else:
        raise ValueError(op)
    return worst / scale_ref, count


CONV_OPS = (A.OP_CONV, A.OP_CONV_DGRAD, A.OP_CONV_WGRAD, A.OP_TCONV, A.OP_TCONV_DGRAD, A.OP_TCONV_WGRAD)
