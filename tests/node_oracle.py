"""What each operation of the library's graph must compute, written with the oracle's layer
arithmetic from the operation contracts in include/lms.h.  Used to check every node of a GPU run
against the oracle applied to the GPU's own inputs of that node (deep nets amplify one-ulp bf16
differences through ReLU decisions, so only this per-node comparison is sharp for them)."""
import numpy as np

from oracle import ops
from paper_1807_02037_amd import abi as A


def _round_bf16(a):
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def eval_node(info, attr, x, out_shape):
    """info: lms_node_info, attr: lms_attr, x: list of input arrays (fp64 / int32) in slot order."""
    op, f = info.op, attr.flags
    nsp = len(out_shape) - 2
    if op == A.OP_CONV:
        y = ops.conv_fwd(x[0], x[1], attr.stride, attr.pad)
        i = 2
        if f & A.F_AFFINE:
            y = ops.affine_fwd(y, x[i], x[i + 1])
            i += 2
        if f & A.F_BIAS:
            y = y + x[i]
            i += 1
        if f & A.F_RES:
            y = y + x[i]
        return ops.relu(y) if f & A.F_RELU else y
    if op in (A.OP_CONV_DGRAD, A.OP_TCONV_DGRAD):
        w, i = x[1], 2
        if op == A.OP_CONV_DGRAD and f & A.F_AFFINE:
            w = _round_bf16(w * x[i])          # the kernel multiplies the filter by the scale and stores it as bf16
            i += 1
        if op == A.OP_CONV_DGRAD:
            y = ops.conv_dgrad(x[0], w, out_shape, attr.stride, attr.pad)
        else:
            y = ops.tconv_dgrad(x[0], w)
        if f & A.F_ADDEND:
            y = y + x[i]
            i += 1
        if f & A.F_MASK:
            y = ops.relu_grad(y, x[i])
        return y
    if op == A.OP_CONV_WGRAD:
        return ops.conv_wgrad(x[0], x[1], tuple(attr.filt[j] for j in range(x[0].ndim - 2)), attr.stride, attr.pad)
    if op == A.OP_TCONV:
        return ops.tconv_fwd(x[0], x[1])
    if op == A.OP_TCONV_WGRAD:
        return ops.tconv_wgrad(x[0], x[1])
    if op == A.OP_MAXPOOL:
        return ops.maxpool_fwd(x[0], attr.filt[0], attr.stride, attr.pad)[0]
    if op == A.OP_MAXPOOL_BWD:
        arg = ops.maxpool_fwd(x[1], attr.filt[0], attr.stride, attr.pad)[1]
        y = ops.maxpool_bwd(x[0], arg, x[1].shape, attr.filt[0], attr.stride, attr.pad)
        return ops.relu_grad(y, x[1]) if f & A.F_MASK else y
    if op == A.OP_GAP:
        return ops.gap_fwd(x[0])
    if op == A.OP_GAP_BWD:
        y = ops.gap_bwd(x[0], out_shape)
        return ops.relu_grad(y, x[1]) if f & A.F_MASK else y
    if op == A.OP_CONCAT:
        return ops.concat(x[0], x[1])
    if op == A.OP_SLICE_C:
        y = x[0][..., attr.c_begin:attr.c_begin + attr.c_count]
        return ops.relu_grad(y, x[1]) if f & A.F_MASK else y
    if op == A.OP_MSE:
        return np.array([ops.mse_fwd(x[0], x[1])])
    if op == A.OP_MSE_GRAD:
        y = ops.mse_bwd(x[0], x[1])
        return ops.relu_grad(y, x[2]) if f & A.F_MASK else y
    if op == A.OP_SOFTMAX_CE:
        return np.array([ops.softmax_ce_fwd(x[0], x[1])])
    if op == A.OP_SOFTMAX_CE_GRAD:
        y = ops.softmax_ce_bwd(x[0], x[1])
        return ops.relu_grad(y, x[2]) if f & A.F_MASK else y
    if op == A.OP_GRAD_SUM:
        ng = len(x) - (1 if f & A.F_MASK else 0)
        y = sum(x[1:ng], x[0])
        return ops.relu_grad(y, x[ng]) if f & A.F_MASK else y
    if op == A.OP_COLSUM:
        return ops.bias_bwd(x[0])
    if op == A.OP_SCALE_COLS:
        return x[0] * x[1]
    if op == A.OP_DOT_COLS:
        return (x[0] * x[1]).reshape(-1, x[0].shape[-1]).sum(axis=0)
    if op in (A.OP_SWAP_OUT, A.OP_SWAP_IN):
        return x[0]
    raise ValueError(op)
