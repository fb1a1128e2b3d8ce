"""ctypes declarations of the C ABI in include/lms.h."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblms.so")

OK, EINVAL, ECYCLE, EBUDGET, EOOM_DEVICE, EOOM_HOST, EHIP = 0, -1, -2, -3, -4, -5, -6
BF16, F32, I32 = 0, 1, 2
VAR_PARAM, VAR_INPUT, VAR_TARGET, VAR_CONST = 0, 1, 2, 3
FWD, BWD, UPD, SWAP = 0, 1, 2, 3
READ, UPDATE, CONTROL = 0, 1, 2
DEVICE, HOST = 0, 1
(OP_VARIABLE, OP_CONV, OP_CONV_DGRAD, OP_CONV_WGRAD, OP_TCONV, OP_TCONV_DGRAD, OP_TCONV_WGRAD, OP_MAXPOOL,
 OP_MAXPOOL_BWD, OP_GAP, OP_GAP_BWD, OP_CONCAT, OP_SLICE_C, OP_MSE, OP_MSE_GRAD, OP_SOFTMAX_CE,
 OP_SOFTMAX_CE_GRAD, OP_GRAD_SUM, OP_COLSUM, OP_SCALE_COLS, OP_DOT_COLS, OP_SWAP_OUT, OP_SWAP_IN, OP_SGD, OP_MOMENTUM) = range(25)
F_RELU, F_AFFINE, F_BIAS, F_RES, F_ADDEND, F_MASK = 1, 2, 4, 8, 16, 32
CHAIN_RULE, DIRECT_ORDER, OWN = 0, 1, 2
X_POISON, X_NO_OVERLAP, X_KEEP_ALL, X_DMA_COPY, X_ENCODE_SWAPS, X_TIMING, X_STAGED_SWAPS = 1, 2, 4, 8, 16, 32, 64
CONV_FWD, CONV_DGRAD, CONV_WGRAD, CONV_WGRAD_BIAS = 0, 1, 2, 3


class Attr(C.Structure):
    _fields_ = [("filt", C.c_int32 * 3), ("stride", C.c_int32), ("pad", C.c_int32), ("flags", C.c_uint32),
                ("cout", C.c_int32), ("c_begin", C.c_int32), ("c_count", C.c_int32), ("ndim_out", C.c_int32),
                ("out_dims", C.c_int64 * 5), ("lr", C.c_float)]


class Params(C.Structure):
    _fields_ = [("n_tensors", C.c_int32), ("lb", C.c_int32), ("ub", C.c_int32), ("ctrld_strategy", C.c_int32),
                ("fuse_swapins", C.c_int32), ("fuse_distance", C.c_int32), ("swap_branches", C.c_int32),
                ("branch_threshold", C.c_int32), ("budget_bytes", C.c_uint64), ("starting_op_names", C.c_char_p),
                ("excl_scopes", C.c_char_p), ("incl_scopes", C.c_char_p), ("excl_types", C.c_uint32), ("incl_types", C.c_uint32),
                ("recompute", C.c_int32), ("recompute_depth", C.c_int32), ("device_tflops", C.c_float), ("hbm_gbs", C.c_float),
                ("link_gbs", C.c_float), ("encoded_swaps", C.c_int32)]


class RewriteStats(C.Structure):
    _fields_ = [("tensors_swapped", C.c_int32), ("swap_outs", C.c_int32), ("swap_ins", C.c_int32),
                ("control_edges", C.c_int32), ("unrewritten", C.c_int32), ("peak_live_before", C.c_uint64),
                ("peak_live_after", C.c_uint64), ("arena_needed_before", C.c_uint64), ("arena_needed_after", C.c_uint64),
                ("swapped_bytes_out", C.c_uint64), ("swapped_bytes_in", C.c_uint64), ("recomputed", C.c_int32), ("estimated_ms", C.c_float)]


class NodeInfo(C.Structure):
    _fields_ = [("id", C.c_int32), ("op", C.c_int32), ("phase", C.c_int32), ("placement", C.c_int32),
                ("is_variable", C.c_int32), ("var_kind", C.c_int32), ("dtype", C.c_int32), ("ndim", C.c_int32),
                ("dims", C.c_int64 * 5), ("gamma", C.c_int32), ("n_inputs", C.c_int32), ("n_control_inputs", C.c_int32),
                ("flags", C.c_uint32), ("bytes", C.c_uint64), ("workspace_bytes", C.c_uint64), ("name", C.c_char * 96)]


class EdgeInfo(C.Structure):
    _fields_ = [("src", C.c_int32), ("dst", C.c_int32), ("action", C.c_int32), ("slot", C.c_int32), ("bytes", C.c_uint64)]


class StepStats(C.Structure):
    _fields_ = [("ms", C.c_float), ("bytes_d2h", C.c_uint64), ("bytes_h2d", C.c_uint64), ("arena_bytes_used", C.c_uint64),
                ("pinned_bytes_used", C.c_uint64), ("n_kernels", C.c_int32), ("n_copies", C.c_int32), ("stall_h2d_ms", C.c_float),
                ("stall_d2h_ms", C.c_float), ("busy_d2h_ms", C.c_float), ("busy_h2d_ms", C.c_float), ("device_ms", C.c_float)]


class ConvDesc(C.Structure):
    _fields_ = [("ndim_sp", C.c_int32), ("n", C.c_int64), ("in_sp", C.c_int64 * 3), ("c", C.c_int32), ("k", C.c_int32),
                ("filt", C.c_int32 * 3), ("stride", C.c_int32), ("pad", C.c_int32), ("flags", C.c_uint32)]


P = C.POINTER
VP = C.c_void_p
_SIGS = {
    "lms_last_error": (C.c_char_p, []),
    "lms_version": (C.c_char_p, []),
    "lms_graph_create": (C.c_int, [P(VP)]),
    "lms_graph_destroy": (C.c_int, [VP]),
    "lms_graph_clone": (C.c_int, [VP, P(VP)]),
    "lms_add_variable": (C.c_int, [VP, C.c_char_p, C.c_int, C.c_int32, P(C.c_int64), C.c_int, P(C.c_int32)]),
    "lms_add_op": (C.c_int, [VP, C.c_char_p, C.c_int, P(Attr), C.c_int32, P(C.c_int32), C.c_int, P(C.c_int32)]),
    "lms_add_update_edge": (C.c_int, [VP, C.c_int32, C.c_int32]),
    "lms_add_control_edge": (C.c_int, [VP, C.c_int32, C.c_int32]),
    "lms_build_backward": (C.c_int, [VP, C.c_int32]),
    "lms_build_update": (C.c_int, [VP, C.c_float, C.c_float, P(C.c_int32)]),
    "lms_params_default": (C.c_int, [P(Params)]),
    "lms_rewrite": (C.c_int, [VP, P(Params), P(RewriteStats)]),
    "lms_memory_need": (C.c_int, [VP, P(C.c_uint64), P(C.c_uint64)]),
    "lms_node_count": (C.c_int, [VP, P(C.c_int32)]),
    "lms_node_info_get": (C.c_int, [VP, C.c_int32, P(NodeInfo)]),
    "lms_node_find": (C.c_int, [VP, C.c_char_p, P(C.c_int32)]),
    "lms_node_set_external": (C.c_int, [VP, C.c_int32, C.c_int32]),
    "lms_node_attr_get": (C.c_int, [VP, C.c_int32, P(Attr)]),
    "lms_edge_count": (C.c_int, [VP, P(C.c_int32)]),
    "lms_edge_info_get": (C.c_int, [VP, C.c_int32, P(EdgeInfo)]),
    "lms_topo_order": (C.c_int, [VP, P(C.c_int32)]),
    "lms_schedule": (C.c_int, [VP, P(C.c_int32)]),
    "lms_exec_create": (C.c_int, [VP, VP, C.c_uint64, VP, C.c_uint64, VP, VP, VP, C.c_uint32, P(VP)]),
    "lms_exec_destroy": (C.c_int, [VP]),
    "lms_pinned_alloc": (C.c_int, [C.c_uint64, P(VP)]),
    "lms_pinned_free": (C.c_int, [VP]),
    "lms_exec_bind": (C.c_int, [VP, C.c_int32, VP]),
    "lms_exec_set_swap_grid": (C.c_int, [VP, C.c_int32, C.c_int32]),
    "lms_exec_step": (C.c_int, [VP, P(C.c_float), P(StepStats)]),
    "lms_exec_tensor_ptr": (C.c_int, [VP, C.c_int32, P(VP)]),
    "lms_conv_workspace_bytes": (C.c_int, [P(ConvDesc), C.c_int32, P(C.c_uint64)]),
    "lms_conv_fwd": (C.c_int, [P(ConvDesc), VP, VP, VP, VP, VP, VP, VP, VP]),
    "lms_conv_dgrad": (C.c_int, [P(ConvDesc), VP, VP, VP, VP, VP, VP, VP, VP]),
    "lms_conv_wgrad": (C.c_int, [P(ConvDesc), VP, VP, VP, VP, VP]),
    "lms_conv_wgrad_bias": (C.c_int, [P(ConvDesc), VP, VP, VP, VP, VP, VP]),
    "lms_static_scratch_bytes": (C.c_uint64, []),
    "lms_conv_wgrad_static": (C.c_int, [P(ConvDesc), VP, VP, VP, VP]),
    "lms_swap_staging_bytes": (C.c_uint64, []),
    "lms_swap_encode_staged": (C.c_int, [VP, VP, C.c_uint64, C.c_int64, C.c_int64, VP, C.c_int32, VP]),
    "lms_swap_decode_staged": (C.c_int, [VP, VP, C.c_uint64, C.c_int64, C.c_int64, VP, C.c_int32, VP]),
    "lms_device_copy": (C.c_int, [VP, VP, C.c_uint64, VP]),
    "lms_mfma_probe": (C.c_int, [C.c_uint32, C.c_int32, C.POINTER(C.c_uint64), VP]),
    "lms_swap_encoded_bytes": (C.c_int, [C.c_uint64, P(C.c_uint64)]),
    "lms_swap_encode": (C.c_int, [VP, VP, C.c_uint64, VP]),
    "lms_swap_decode": (C.c_int, [VP, VP, C.c_uint64, VP]),
    "lms_swap_moved_bytes": (C.c_int, [VP, C.c_uint64, P(C.c_uint64)]),
}
EXPORTS = sorted(_SIGS)

_lib = None


def lib():
    """The loaded library.  Fails loudly if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1807_02037_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        # PyTorch supplies device memory and streams, and ships its own HIP runtime: it has to be in the
        # process first so that this library binds to the same runtime instead of loading a second one
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib
