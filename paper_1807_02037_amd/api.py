"""Python names for the calls of include/lms.h (marshalling only)."""
import ctypes as C

from . import _lib as A


class LmsError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"lms status {status}: {msg}")
        self.status = status


def _ck(st):
    if st != A.OK:
        raise LmsError(st, A.lib().lms_last_error().decode())


_NAME_LISTS = {"starting_op_names": "starting_op_names", "starting_op_name": "starting_op_names",
               "excl_scopes": "excl_scopes", "excl_scope": "excl_scopes", "incl_scopes": "incl_scopes", "incl_scope": "incl_scopes"}
_TYPE_LISTS = {"excl_types": "excl_types", "excl_type": "excl_types", "incl_types": "incl_types", "incl_type": "incl_types"}


def params(**kw):
    """lms_params with the defaults of Table 2, overridden by keyword.  The list-valued fields of Table 2 take a
    single value or a sequence: names are joined with commas, operation types become a bit mask."""
    p = A.Params()
    _ck(A.lib().lms_params_default(C.byref(p)))
    for k, v in kw.items():
        if k in _NAME_LISTS:
            names = [v] if isinstance(v, (str, bytes)) else list(v or ())
            names = [n.decode() if isinstance(n, bytes) else n for n in names]
            assert not any("," in n for n in names), "names in a list must not contain a comma"
            setattr(p, _NAME_LISTS[k], ",".join(names).encode() if names else None)
            continue
        if k in _TYPE_LISTS:
            ops = [v] if isinstance(v, int) else list(v or ())
            setattr(p, _TYPE_LISTS[k], sum(1 << o for o in set(ops) if o >= 0))
            continue
        if isinstance(v, str):
            v = v.encode()
        if not hasattr(p, k):
            raise AttributeError(k)
        setattr(p, k, v)
    return p


class Graph:
    """lms_graph handle."""

    def __init__(self, handle=None):
        if handle is None:
            handle = C.c_void_p()
            _ck(A.lib().lms_graph_create(C.byref(handle)))
        self.h = handle

    def __del__(self):
        if getattr(self, "h", None) is not None and A._lib is not None:
            A._lib.lms_graph_destroy(self.h)
            self.h = None

    def clone(self):
        out = C.c_void_p()
        _ck(A.lib().lms_graph_clone(self.h, C.byref(out)))
        return Graph(out)

    def add_variable(self, name, dtype, dims, kind):
        out = C.c_int32()
        arr = (C.c_int64 * len(dims))(*dims)
        _ck(A.lib().lms_add_variable(self.h, name.encode(), dtype, len(dims), arr, kind, C.byref(out)))
        return out.value

    def add_op(self, name, op, inputs, phase=A.FWD, **attr):
        a = A.Attr()
        a.filt[0] = a.filt[1] = a.filt[2] = 1
        a.stride = 1
        for k, v in attr.items():
            if k == "filt":
                for i, f in enumerate(v):
                    a.filt[i] = f
            elif k == "out_dims":
                a.ndim_out = len(v)
                for i, d in enumerate(v):
                    a.out_dims[i] = d
            else:
                setattr(a, k, v)
        out = C.c_int32()
        arr = (C.c_int32 * len(inputs))(*inputs)
        _ck(A.lib().lms_add_op(self.h, name.encode(), op, C.byref(a), len(inputs), arr, phase, C.byref(out)))
        return out.value

    def add_update_edge(self, src, var):
        _ck(A.lib().lms_add_update_edge(self.h, src, var))

    def add_control_edge(self, src, dst):
        _ck(A.lib().lms_add_control_edge(self.h, src, dst))

    def build_backward(self, loss_node):
        _ck(A.lib().lms_build_backward(self.h, loss_node))

    def build_update(self, lr, momentum=0.0):
        n = C.c_int32()
        _ck(A.lib().lms_build_update(self.h, lr, momentum, C.byref(n)))
        return n.value

    def rewrite(self, p=None, **kw):
        p = p if p is not None else params(**kw)
        st = A.RewriteStats()
        _ck(A.lib().lms_rewrite(self.h, C.byref(p), C.byref(st)))
        return st

    def memory_need(self):
        a, b = C.c_uint64(), C.c_uint64()
        _ck(A.lib().lms_memory_need(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def node_count(self):
        n = C.c_int32()
        _ck(A.lib().lms_node_count(self.h, C.byref(n)))
        return n.value

    def node_info(self, i):
        info = A.NodeInfo()
        _ck(A.lib().lms_node_info_get(self.h, i, C.byref(info)))
        return info

    def set_external(self, i, external=True):
        """The output of node i will be bound to caller memory: no arena block is planned for it."""
        _ck(A.lib().lms_node_set_external(self.h, i, 1 if external else 0))

    def node_attr(self, i):
        a = A.Attr()
        _ck(A.lib().lms_node_attr_get(self.h, i, C.byref(a)))
        return a

    def node_inputs(self, i):
        """Data inputs of node i in slot order."""
        es = sorted((e.slot, e.src) for e in self.edges() if e.dst == i and e.action == A.READ)
        return [src for _, src in es]

    def find(self, name):
        out = C.c_int32()
        _ck(A.lib().lms_node_find(self.h, name.encode(), C.byref(out)))
        return out.value

    def edges(self):
        n = C.c_int32()
        _ck(A.lib().lms_edge_count(self.h, C.byref(n)))
        out = []
        for i in range(n.value):
            e = A.EdgeInfo()
            _ck(A.lib().lms_edge_info_get(self.h, i, C.byref(e)))
            out.append(e)
        return out

    def topo_order(self):
        n = self.node_count()
        arr = (C.c_int32 * n)()
        _ck(A.lib().lms_topo_order(self.h, arr))
        return list(arr)

    def schedule(self):
        n = self.node_count()
        arr = (C.c_int32 * n)()
        _ck(A.lib().lms_schedule(self.h, arr))
        return list(arr)


class PinnedPool:
    """Pinned host memory of exactly nbytes (lms_pinned_alloc), freed with the object."""

    def __init__(self, nbytes):
        p = C.c_void_p()
        _ck(A.lib().lms_pinned_alloc(int(nbytes), C.byref(p)))
        self.ptr, self.nbytes = p.value, int(nbytes)

    def free(self):
        if getattr(self, "ptr", None) and A._lib is not None:
            A._lib.lms_pinned_free(self.ptr)
        self.ptr = None

    __del__ = free


class Executor:
    """lms_exec handle.  arena / pinned / streams are raw addresses owned by the caller."""

    def __init__(self, graph, arena_ptr, arena_bytes, pinned_ptr, pinned_bytes, compute, d2h, h2d, flags=0):
        self.h = C.c_void_p()
        self.graph = graph
        _ck(A.lib().lms_exec_create(graph.h, arena_ptr, arena_bytes, pinned_ptr, pinned_bytes, compute, d2h, h2d,
                                    flags, C.byref(self.h)))

    def __del__(self):
        if getattr(self, "h", None) and A._lib is not None:
            A._lib.lms_exec_destroy(self.h)
            self.h = None

    def bind(self, node, device_ptr):
        _ck(A.lib().lms_exec_bind(self.h, node, device_ptr))

    def set_swap_grid(self, encode_workgroups=0, decode_workgroups=0):
        _ck(A.lib().lms_exec_set_swap_grid(self.h, encode_workgroups, decode_workgroups))

    def step(self, sync=True):
        st = A.StepStats()
        loss = C.c_float()
        _ck(A.lib().lms_exec_step(self.h, C.byref(loss) if sync else None, C.byref(st)))
        return (loss.value if sync else None), st

    def tensor_ptr(self, node):
        p = C.c_void_p()
        _ck(A.lib().lms_exec_tensor_ptr(self.h, node, C.byref(p)))
        return p.value


def conv_desc(n, in_sp, c, k, filt, stride=1, pad=0, flags=0):
    d = A.ConvDesc()
    d.ndim_sp = len(in_sp)
    d.n, d.c, d.k, d.stride, d.pad, d.flags = n, c, k, stride, pad, flags
    for i in range(3):
        d.in_sp[i] = in_sp[i] if i < len(in_sp) else 1
        d.filt[i] = filt[i] if i < len(filt) else 1
    return d


def conv_workspace_bytes(desc, which):
    out = C.c_uint64()
    _ck(A.lib().lms_conv_workspace_bytes(C.byref(desc), which, C.byref(out)))
    return out.value


def conv_fwd(desc, x, w, scale, shift, res, y, workspace, stream):
    _ck(A.lib().lms_conv_fwd(C.byref(desc), x, w, scale, shift, res, y, workspace, stream))


def conv_dgrad(desc, dy, w, scale, addend, mask, dx, workspace, stream):
    _ck(A.lib().lms_conv_dgrad(C.byref(desc), dy, w, scale, addend, mask, dx, workspace, stream))


def conv_wgrad(desc, x, dy, dw, workspace, stream):
    _ck(A.lib().lms_conv_wgrad(C.byref(desc), x, dy, dw, workspace, stream))


def conv_wgrad_bias(desc, x, dy, dw, dbias, workspace, stream):
    _ck(A.lib().lms_conv_wgrad_bias(C.byref(desc), x, dy, dw, dbias, workspace, stream))


def swap_encode_staged(dst_host, src, numel, slot_begin, slot_end, stage, w, stream):
    _ck(A.lib().lms_swap_encode_staged(dst_host, src, numel, slot_begin, slot_end, stage, w, stream))


def swap_decode_staged(dst, src_host, numel, slot_begin, slot_end, stage, w, stream):
    _ck(A.lib().lms_swap_decode_staged(dst, src_host, numel, slot_begin, slot_end, stage, w, stream))


def swap_staging_bytes():
    """Arena bytes that X_STAGED_SWAPS takes for its staging buffers (rewrite for budget - this)."""
    return int(A.lib().lms_swap_staging_bytes())


def conv_wgrad_static(desc, x, dy, dw, stream):
    _ck(A.lib().lms_conv_wgrad_static(C.byref(desc), x, dy, dw, stream))


def static_scratch_bytes():
    return A.lib().lms_static_scratch_bytes()


def swap_encoded_bytes(numel):
    b = C.c_uint64()
    _ck(A.lib().lms_swap_encoded_bytes(numel, C.byref(b)))
    return b.value


def swap_encode(dst_host, src, numel, stream):
    _ck(A.lib().lms_swap_encode(dst_host, src, numel, stream))


def swap_decode(dst, src_host, numel, stream):
    _ck(A.lib().lms_swap_decode(dst, src_host, numel, stream))


def swap_moved_bytes(host, numel):
    b = C.c_uint64()
    _ck(A.lib().lms_swap_moved_bytes(host, numel, C.byref(b)))
    return b.value
