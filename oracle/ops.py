"""Reference arithmetic of one CNN training step, fp64, channels-last.

TEST INFRASTRUCTURE ONLY: a plain, slow CPU statement of what the layers of
the training step compute.  Nothing in the product path may import it.

The paper does not define layer arithmetic (it only says training is mostly
matrix multiplication, Section 1, and that a backward function of layer i
needs layer i's forward output, Section 3.3), so each function below is the
textbook definition of the operation, written out tap by tap with a matrix
product over channels as the only library step.  Activations are
(N, spatial..., C); filters are (filter spatial..., C, K).
"""
import numpy as np


def _out_len(h, r, stride, pad):
    return (h + 2 * pad - r) // stride + 1


def _pad_spatial(x, pad, value=0.0):
    if pad == 0:
        return x
    nd = x.ndim - 2
    return np.pad(x, [(0, 0)] + [(pad, pad)] * nd + [(0, 0)], constant_values=value)


def _tap_slices(tap, out_sp, stride):
    # positions o*stride + tap for o = 0..O-1 along every spatial axis (in padded coordinates)
    return (slice(None),) + tuple(slice(tap[i], tap[i] + (out_sp[i] - 1) * stride + 1, stride)
                                  for i in range(len(tap)))


def conv_fwd(x, w, stride=1, pad=0):
    """Cross-correlation with zero padding:
    y[n,o,k] = sum_{r,c} x[n, o*stride + r - pad, c] * w[r,c,k]  (o, r multi-indices)."""
    nd = x.ndim - 2
    filt = w.shape[:nd]
    out_sp = tuple(_out_len(x.shape[1 + i], filt[i], stride, pad) for i in range(nd))
    xp = _pad_spatial(x, pad)
    y = np.zeros((x.shape[0],) + out_sp + (w.shape[-1],), dtype=np.float64)
    for tap in np.ndindex(*filt):
        y += xp[_tap_slices(tap, out_sp, stride)] @ w[tap]
    return y


def conv_dgrad(dy, w, x_shape, stride=1, pad=0):
    """Gradient of conv_fwd w.r.t. x: every output position o sends dy[n,o,:] @ w[r]^T
    back to input position o*stride + r - pad."""
    nd = dy.ndim - 2
    filt = w.shape[:nd]
    out_sp = dy.shape[1:-1]
    padded = (x_shape[0],) + tuple(x_shape[1 + i] + 2 * pad for i in range(nd)) + (x_shape[-1],)
    dxp = np.zeros(padded, dtype=np.float64)
    for tap in np.ndindex(*filt):
        dxp[_tap_slices(tap, out_sp, stride)] += dy @ w[tap].T
    if pad == 0:
        return dxp
    crop = (slice(None),) + tuple(slice(pad, pad + x_shape[1 + i]) for i in range(nd))
    return np.ascontiguousarray(dxp[crop])


def conv_wgrad(x, dy, filt, stride=1, pad=0):
    """Gradient of conv_fwd w.r.t. w: dw[r,c,k] = sum_{n,o} x[n, o*stride + r - pad, c] * dy[n,o,k]."""
    out_sp = dy.shape[1:-1]
    xp = _pad_spatial(x, pad)
    dw = np.zeros(tuple(filt) + (x.shape[-1], dy.shape[-1]), dtype=np.float64)
    dy2 = dy.reshape(-1, dy.shape[-1])
    for tap in np.ndindex(*filt):
        xs = xp[_tap_slices(tap, out_sp, stride)].reshape(-1, x.shape[-1])
        dw[tap] = xs.T @ dy2
    return dw


def tconv_fwd(x, w):
    """Transposed convolution, window 2 and stride 2 in every spatial axis (non-overlapping):
    y[n, 2*d + i, k] = sum_c x[n,d,c] * w[i,c,k]."""
    nd = x.ndim - 2
    y = np.zeros((x.shape[0],) + tuple(2 * s for s in x.shape[1:-1]) + (w.shape[-1],), dtype=np.float64)
    for tap in np.ndindex(*(2,) * nd):
        y[(slice(None),) + tuple(slice(t, None, 2) for t in tap)] = x @ w[tap]
    return y


def tconv_dgrad(dy, w):
    nd = dy.ndim - 2
    dx = np.zeros((dy.shape[0],) + tuple(s // 2 for s in dy.shape[1:-1]) + (w.shape[-2],), dtype=np.float64)
    for tap in np.ndindex(*(2,) * nd):
        dx += dy[(slice(None),) + tuple(slice(t, None, 2) for t in tap)] @ w[tap].T
    return dx


def tconv_wgrad(x, dy):
    nd = x.ndim - 2
    dw = np.zeros((2,) * nd + (x.shape[-1], dy.shape[-1]), dtype=np.float64)
    x2 = x.reshape(-1, x.shape[-1])
    for tap in np.ndindex(*(2,) * nd):
        d = dy[(slice(None),) + tuple(slice(t, None, 2) for t in tap)]
        dw[tap] = x2.T @ d.reshape(-1, dy.shape[-1])
    return dw


def relu(x):
    return np.maximum(x, 0.0)


def relu_grad(dy, y):
    """Derivative taken as 0 at y == 0."""
    return dy * (y > 0.0)


def affine_fwd(x, scale, shift):
    """Per-channel y = scale_c * x + shift_c."""
    return x * scale + shift


def affine_bwd(dy, x, scale):
    """Returns (dx, dscale, dshift)."""
    red = tuple(range(dy.ndim - 1))
    return dy * scale, (dy * x).sum(axis=red), dy.sum(axis=red)


def bias_bwd(dy):
    return dy.sum(axis=tuple(range(dy.ndim - 1)))


def maxpool_fwd(x, win, stride, pad=0):
    """Window maximum (padding counts as -inf).  Also returns, per output element, the
    row-major window index of the FIRST maximal element, which receives the gradient."""
    nd = x.ndim - 2
    out_sp = tuple(_out_len(x.shape[1 + i], win, stride, pad) for i in range(nd))
    xp = _pad_spatial(x, pad, -np.inf)
    best = np.full((x.shape[0],) + out_sp + (x.shape[-1],), -np.inf)
    arg = np.zeros(best.shape, dtype=np.int64)
    for t, tap in enumerate(np.ndindex(*(win,) * nd)):
        v = xp[_tap_slices(tap, out_sp, stride)]
        better = v > best            # strict: ties stay with the earlier window element
        best = np.where(better, v, best)
        arg = np.where(better, t, arg)
    return best, arg


def maxpool_bwd(dy, arg, x_shape, win, stride, pad=0):
    nd = dy.ndim - 2
    out_sp = dy.shape[1:-1]
    padded = (x_shape[0],) + tuple(x_shape[1 + i] + 2 * pad for i in range(nd)) + (x_shape[-1],)
    dxp = np.zeros(padded, dtype=np.float64)
    for t, tap in enumerate(np.ndindex(*(win,) * nd)):
        dxp[_tap_slices(tap, out_sp, stride)] += dy * (arg == t)
    if pad == 0:
        return dxp
    crop = (slice(None),) + tuple(slice(pad, pad + x_shape[1 + i]) for i in range(nd))
    return np.ascontiguousarray(dxp[crop])


def gap_fwd(x):
    """Mean over all spatial positions; spatial axes kept with length 1."""
    return x.mean(axis=tuple(range(1, x.ndim - 1)), keepdims=True)


def gap_bwd(dy, x_shape):
    count = int(np.prod(x_shape[1:-1]))
    return np.broadcast_to(dy / count, x_shape).copy()


def concat(a, b):
    return np.concatenate([a, b], axis=-1)


def concat_bwd(dy, ca):
    return np.ascontiguousarray(dy[..., :ca]), np.ascontiguousarray(dy[..., ca:])


def mse_fwd(y, t):
    """Mean over ALL elements (batch included) of (y - t)^2."""
    d = y - t
    return float((d * d).sum() / d.size)


def mse_bwd(y, t):
    return 2.0 * (y - t) / y.size


def softmax_ce_fwd(z, labels):
    """Mean over rows (all leading axes) of -log softmax(z)[label]; log-sum-exp with max subtraction."""
    z2 = z.reshape(-1, z.shape[-1])
    lab = labels.reshape(-1)
    m = z2.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(z2 - m).sum(axis=1))
    return float((lse - z2[np.arange(z2.shape[0]), lab]).sum() / z2.shape[0])


def softmax_ce_bwd(z, labels):
    z2 = z.reshape(-1, z.shape[-1])
    lab = labels.reshape(-1)
    e = np.exp(z2 - z2.max(axis=1, keepdims=True))
    p = e / e.sum(axis=1, keepdims=True)
    p[np.arange(z2.shape[0]), lab] -= 1.0
    return (p / z2.shape[0]).reshape(z.shape)
