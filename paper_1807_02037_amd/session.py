"""Plumbing around one executor: device arena and streams come from PyTorch, the pinned pool from the library, every
step of the training pass runs inside liblms.so."""
import numpy as np
import torch

from . import _lib as A
from .api import Executor, PinnedPool, swap_encoded_bytes, swap_staging_bytes
from .models import build_graph


def to_device(arr, dtype):
    """Host array -> device tensor of the library's storage type (values must be representable).
    A tensor that already sits on the device in that type is used as it is."""
    want = {A.BF16: torch.bfloat16, A.F32: torch.float32}.get(dtype, torch.int32)
    if isinstance(arr, torch.Tensor):
        assert arr.is_cuda and arr.dtype == want and arr.is_contiguous()
        return arr
    if dtype == A.BF16:
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(torch.bfloat16).cuda()
    if dtype == A.F32:
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.int32)).cuda()


class Session:
    """Builds the graph of a workload, optionally rewrites it, and owns the memory the executor runs in."""

    def __init__(self, spec, tensors, rewrite=None, arena_bytes=None, flags=0, dtype=A.BF16, lr=None, backward=True, momentum=0.0):
        self.spec = spec
        self.g, self.ids = build_graph(spec, backward=backward, dtype=dtype, lr=lr, momentum=momentum)
        self.unswapped_need = self.g.memory_need()[1]
        self.rewrite_stats = None
        if rewrite is not None:
            self.rewrite_stats = self.g.rewrite(**rewrite)
        self.infos = [self.g.node_info(i) for i in range(self.g.node_count())]
        need = self.g.memory_need()[1]
        if flags & A.X_KEEP_ALL:
            need = sum((i.bytes + 255) // 256 * 256 + (i.workspace_bytes + 255) // 256 * 256
                       for i in self.infos if not i.is_variable)
        encode = bool(flags & A.X_ENCODE_SWAPS) and not (flags & A.X_DMA_COPY)
        if encode and (flags & A.X_STAGED_SWAPS) and arena_bytes is None:
            need += swap_staging_bytes()        # the staging buffers take the end of the arena
        self.arena_bytes = int(arena_bytes if arena_bytes is not None else need)

        def host_bytes(i):
            numel = i.bytes // 2
            if encode and i.dtype == A.BF16 and numel and numel % 8 == 0:
                return swap_encoded_bytes(numel)
            return i.bytes
        pinned = sum((host_bytes(i) + 255) // 256 * 256 for i in self.infos if i.op == A.OP_SWAP_OUT)
        self.arena = torch.empty(max(self.arena_bytes, 256), dtype=torch.uint8, device="cuda")
        # the pool comes from the library: PyTorch's pinned allocator rounds sizes up to a power of two
        self.pinned = PinnedPool(max(pinned, 256))
        self.streams = [torch.cuda.Stream() for _ in range(3)]
        self.ex = Executor(self.g, self.arena.data_ptr(), self.arena_bytes, self.pinned.ptr, pinned,
                           *[s.cuda_stream for s in self.streams], flags)
        self.dev = {}
        for info in self.infos:
            name = info.name.decode()
            if info.is_variable:
                if name.startswith("velocity/"):         # optimiser state: starts at zero
                    t = torch.zeros(tuple(info.dims[i] for i in range(info.ndim)), dtype=torch.float32, device="cuda")
                else:
                    t = to_device(tensors[name], info.dtype)
                assert t.numel() * t.element_size() == info.bytes, name
                self.dev[name] = t
                self.ex.bind(info.id, t.data_ptr())
            elif name.startswith("grad/"):
                t = torch.zeros(tuple(info.dims[i] for i in range(info.ndim)), dtype=torch.float32, device="cuda")
                self.dev[name] = t
                self.ex.bind(info.id, t.data_ptr())
        # update operations write into the parameter they update: the step trains in place
        for info in self.infos:
            name = info.name.decode()
            if name.startswith("update/"):
                self.ex.bind(info.id, self.dev[name[len("update/"):]].data_ptr())
        torch.cuda.synchronize()

    def __del__(self):
        # the executor goes before the memory it runs in
        self.ex = None
        if getattr(self, "pinned", None) is not None:
            self.pinned.free()

    def param(self, name):
        """Current value of a bound variable (fp64 array)."""
        torch.cuda.synchronize()
        return self.dev[name].float().cpu().numpy().astype(np.float64)

    def step(self, sync=True):
        return self.ex.step(sync)

    def grads(self):
        torch.cuda.synchronize()
        return {k: v.cpu().numpy().astype(np.float64) for k, v in self.dev.items() if k.startswith("grad/")}

    def grad_bits(self):
        torch.cuda.synchronize()
        return {k: v.cpu().numpy().view(np.uint32).copy() for k, v in self.dev.items() if k.startswith("grad/")}

    def activation(self, name):
        """Value of a named node's output after a synchronised step (meaningful with X_KEEP_ALL)."""
        return self.node_value(self.ids[name])

    def node_tensor(self, node):
        """Any node's output as a device tensor in its storage type (a view of the bound tensor or of the arena)."""
        info = self.infos[node]
        name = info.name.decode()
        if name in self.dev:
            return self.dev[name]
        off = self.ex.tensor_ptr(info.id) - self.arena.data_ptr()
        dt = {A.BF16: torch.bfloat16, A.F32: torch.float32, A.I32: torch.int32}[info.dtype]
        shape = tuple(info.dims[i] for i in range(info.ndim))
        return self.arena[off:off + info.bytes].view(dt).reshape(shape)

    def node_value(self, node):
        """Value of any node's output (variable, bound gradient or arena tensor) as fp64 / int32."""
        torch.cuda.synchronize()
        info = self.infos[node]
        name = info.name.decode()
        if name in self.dev:
            t = self.dev[name]
            return t.cpu().numpy() if info.dtype == A.I32 else t.float().cpu().numpy().astype(np.float64)
        off = self.ex.tensor_ptr(info.id) - self.arena.data_ptr()
        raw = self.arena[off:off + info.bytes]
        dt = {A.BF16: torch.bfloat16, A.F32: torch.float32, A.I32: torch.int32}[info.dtype]
        shape = tuple(info.dims[i] for i in range(info.ndim))
        return raw.view(dt).reshape(shape).float().cpu().numpy().astype(np.float64)
