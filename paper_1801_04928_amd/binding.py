"""ctypes binding of liblf.so: one Python function per C entry point of include/lf.h, same names,
plus `LeapfrogNet`, a convenience owner of the device buffers (torch tensors) around one handle.

There is no fallback: if the library has not been built, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

LF_OK, LF_EINVAL, LF_ESTATE, LF_ENOMEM, LF_EHIP, LF_EUNSUPPORTED = range(6)
LF_F32, LF_BF16 = 0, 1
LF_COST_QUADRATIC = 0
LF_SCHED_AUTO, LF_SCHED_STREAMS, LF_SCHED_PERSISTENT, LF_SCHED_REDUNDANT, LF_SCHED_FUSED = 0, 1, 2, 3, 4
LF_DEBUG_CHAIN_ONLY = 1

_STATUS_NAMES = {0: "LF_OK", 1: "LF_EINVAL", 2: "LF_ESTATE", 3: "LF_ENOMEM", 4: "LF_EHIP", 5: "LF_EUNSUPPORTED"}


class LfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


def library_path() -> str:
    return os.path.join(HERE, "liblf.so")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_1801_04928_amd.build)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_1801_04928_amd.build`")
        # PyTorch brings a HIP runtime of its own; the library must bind to that same runtime, not to a second
        # copy loaded before it (two runtimes in one process do not share a device context), so torch goes first.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(path)
        vp, vpp, i, sz = C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_size_t
        L.lf_workspace_bytes.restype, L.lf_workspace_bytes.argtypes = sz, [i, i, i, i]
        L.lf_create.restype, L.lf_create.argtypes = i, [vpp, i, i, i, i, i, vp, sz]
        ip = C.POINTER(C.c_int)
        L.lf_workspace_bytes_widths.restype, L.lf_workspace_bytes_widths.argtypes = sz, [i, ip, i, i]
        L.lf_create_widths.restype, L.lf_create_widths.argtypes = i, [vpp, i, ip, i, i, i, vp, sz]
        L.lf_set_params.restype, L.lf_set_params.argtypes = i, [vp, vpp, vpp]
        L.lf_set_grad_buffers.restype, L.lf_set_grad_buffers.argtypes = i, [vp, vpp, vpp]
        L.lf_set_schedule.restype, L.lf_set_schedule.argtypes = i, [vp, i]
        L.lf_set_debug_flags.restype, L.lf_set_debug_flags.argtypes = i, [vp, C.c_uint]
        L.lf_set_cost_scale.restype, L.lf_set_cost_scale.argtypes = i, [vp, i]
        L.lf_set_sgd.restype, L.lf_set_sgd.argtypes = i, [vp, C.c_float]
        L.lf_set_master_weights.restype, L.lf_set_master_weights.argtypes = i, [vp, vpp]
        L.lf_forward.restype, L.lf_forward.argtypes = i, [vp, vp, vp]
        L.lf_backward_leapfrog.restype, L.lf_backward_leapfrog.argtypes = i, [vp, vp, i, vp]
        L.lf_backward_leapfrog_noalloc.restype, L.lf_backward_leapfrog_noalloc.argtypes = i, [vp, vp, i, vp]
        L.lf_noalloc_scratch_limit.restype, L.lf_noalloc_scratch_limit.argtypes = sz, []
        L.lf_grads.restype, L.lf_grads.argtypes = i, [vp, i, vpp, vpp]
        L.lf_activations.restype, L.lf_activations.argtypes = i, [vp, i, vpp, vpp]
        L.lf_schedule_worker.restype, L.lf_schedule_worker.argtypes = i, [i, i, i]
        L.lf_algorithm1_owner.restype, L.lf_algorithm1_owner.argtypes = i, [i, i, i]
        L.lf_last_error.restype, L.lf_last_error.argtypes = C.c_char_p, [vp]
        L.lf_destroy.restype, L.lf_destroy.argtypes = None, [vp]
        _lib = L
    return _lib


def _ptr_array(ptrs: Optional[Sequence[int]]):
    if ptrs is None:
        return None
    return (C.c_void_p * len(ptrs))(*ptrs)


# ---- thin functions, same names and argument order as the C ABI; they return the lf_status ----------
def lf_workspace_bytes(L: int, N: int, B: int, dt: int) -> int:
    return int(lib().lf_workspace_bytes(L, N, B, dt))


def lf_create(L: int, N: int, B: int, dt: int, cost: int, workspace: int, workspace_bytes: int):
    """Returns (status, handle); handle is None unless status == LF_OK."""
    h = C.c_void_p()
    st = lib().lf_create(C.byref(h), L, N, B, dt, cost, C.c_void_p(workspace), workspace_bytes)
    return st, (h if st == LF_OK else None)


def _int_array(values: Optional[Sequence[int]]):
    if values is None:
        return None
    return (C.c_int * len(values))(*values)


def lf_workspace_bytes_widths(L: int, n: Optional[Sequence[int]], B: int, dt: int) -> int:
    return int(lib().lf_workspace_bytes_widths(L, _int_array(n), B, dt))


def lf_create_widths(L: int, n: Optional[Sequence[int]], B: int, dt: int, cost: int, workspace: int,
                     workspace_bytes: int):
    """Returns (status, handle); handle is None unless status == LF_OK."""
    h = C.c_void_p()
    st = lib().lf_create_widths(C.byref(h), L, _int_array(n), B, dt, cost, C.c_void_p(workspace), workspace_bytes)
    return st, (h if st == LF_OK else None)


def lf_set_params(net, w: Optional[Sequence[int]], b: Optional[Sequence[int]]) -> int:
    return lib().lf_set_params(net, _ptr_array(w), _ptr_array(b))


def lf_set_grad_buffers(net, nabla_w: Optional[Sequence[int]], nabla_b: Optional[Sequence[int]]) -> int:
    return lib().lf_set_grad_buffers(net, _ptr_array(nabla_w), _ptr_array(nabla_b))


def lf_set_schedule(net, sched: int) -> int:
    return lib().lf_set_schedule(net, sched)


def lf_set_debug_flags(net, flags: int) -> int:
    return lib().lf_set_debug_flags(net, flags)


def lf_set_cost_scale(net, log2_scale: int) -> int:
    return lib().lf_set_cost_scale(net, log2_scale)


def lf_set_sgd(net, eta: float) -> int:
    return lib().lf_set_sgd(net, eta)


def lf_set_master_weights(net, w32: Optional[Sequence[int]]) -> int:
    return lib().lf_set_master_weights(net, _ptr_array(w32))


def lf_forward(net, x1: int, hip_stream: int = 0) -> int:
    return lib().lf_forward(net, C.c_void_p(x1), C.c_void_p(hip_stream))


def lf_backward_leapfrog(net, y: int, k: int, hip_stream: int = 0) -> int:
    return lib().lf_backward_leapfrog(net, C.c_void_p(y), k, C.c_void_p(hip_stream))


def lf_backward_leapfrog_noalloc(net, y: int, k: int, hip_stream: int = 0) -> int:
    return lib().lf_backward_leapfrog_noalloc(net, C.c_void_p(y), k, C.c_void_p(hip_stream))


def lf_noalloc_scratch_limit() -> int:
    return int(lib().lf_noalloc_scratch_limit())


def lf_grads(net, l: int):
    """Returns (status, nabla_w device pointer, nabla_b device pointer)."""
    pw, pb = C.c_void_p(), C.c_void_p()
    st = lib().lf_grads(net, l, C.byref(pw), C.byref(pb))
    return st, pw.value, pb.value


def lf_activations(net, l: int):
    """Returns (status, a^l device pointer, delta^l device pointer)."""
    pa, pd = C.c_void_p(), C.c_void_p()
    st = lib().lf_activations(net, l, C.byref(pa), C.byref(pd))
    return st, pa.value, pd.value


def lf_schedule_worker(L: int, k: int, l: int) -> int:
    return lib().lf_schedule_worker(L, k, l)


def lf_algorithm1_owner(L: int, k: int, l: int) -> int:
    return lib().lf_algorithm1_owner(L, k, l)


def lf_last_error(net=None) -> str:
    return lib().lf_last_error(net).decode()


def lf_destroy(net) -> None:
    lib().lf_destroy(net)


# ---- convenience owner ---------------------------------------------------------------------------
class LeapfrogNet:
    """Holds the torch tensors (weights, biases, gradients, workspace) of one net on the GPU and the
    library handle that works on them.  Layer indices are the paper's: 2..L.  N is the number of neurons of
    every layer, or a sequence of L widths (layer 1 first)."""

    def __init__(self, L: int, N, B: int = 1, dtype: str = "f32", device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.widths = [int(N)] * L if isinstance(N, int) else [int(v) for v in N]
        if len(self.widths) != L:
            raise LfError(LF_EINVAL, "need one width per layer")
        self.L, self.N, self.B, self.dtype = L, max(self.widths), B, dtype
        self.device = torch.device(device)
        self.dt = {"f32": LF_F32, "bf16": LF_BF16}[dtype]
        self.tdtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        n = self.widths
        if isinstance(N, int):
            nbytes = lf_workspace_bytes(L, N, B, self.dt)
        else:
            nbytes = lf_workspace_bytes_widths(L, n, B, self.dt)
        if nbytes == 0:
            raise LfError(LF_EINVAL, "invalid shape")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        if isinstance(N, int):
            st, self.handle = lf_create(L, N, B, self.dt, LF_COST_QUADRATIC, self.workspace.data_ptr(), nbytes)
        else:
            st, self.handle = lf_create_widths(L, n, B, self.dt, LF_COST_QUADRATIC, self.workspace.data_ptr(),
                                               nbytes)
        if st != LF_OK:
            raise LfError(st, lf_last_error(None))
        dev, f32 = self.device, torch.float32
        self.w = [torch.empty((n[l - 1], n[l - 2]), dtype=self.tdtype, device=dev) for l in range(2, L + 1)]
        self.b = [torch.empty(n[l - 1], dtype=f32, device=dev) for l in range(2, L + 1)]
        self.nabla_w = [torch.empty((n[l - 1], n[l - 2]), dtype=f32, device=dev) for l in range(2, L + 1)]
        self.nabla_b = [torch.empty(n[l - 1], dtype=f32, device=dev) for l in range(2, L + 1)]
        self.x = torch.empty((B, n[0]), dtype=self.tdtype, device=dev)
        self.y = torch.empty((B, n[L - 1]), dtype=self.tdtype, device=dev)
        self.master_w = None
        self._check(lf_set_params(self.handle, [t.data_ptr() for t in self.w], [t.data_ptr() for t in self.b]))
        self._check(lf_set_grad_buffers(self.handle, [t.data_ptr() for t in self.nabla_w],
                                        [t.data_ptr() for t in self.nabla_b]))

    def _check(self, st: int) -> None:
        if st != LF_OK:
            raise LfError(st, lf_last_error(self.handle))

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def load(self, net) -> None:
        """Copy the tensors of an lf_inputs.SyntheticNet (fp32 numpy arrays) to the device."""
        t = self.torch
        for l in range(2, self.L + 1):
            self.w[l - 2].copy_(t.from_numpy(net.w(l)))
            self.b[l - 2].copy_(t.from_numpy(net.b(l)))
            if self.master_w is not None:
                self.master_w[l - 2].copy_(t.from_numpy(net.w(l)))
        self.x.copy_(t.from_numpy(net.x()))
        self.y.copy_(t.from_numpy(net.y()))

    def set_schedule(self, sched: int) -> None:
        self._check(lf_set_schedule(self.handle, sched))

    def set_debug_flags(self, flags: int) -> None:
        self._check(lf_set_debug_flags(self.handle, flags))

    def set_cost_scale(self, log2_scale: int) -> None:
        self._check(lf_set_cost_scale(self.handle, log2_scale))

    def set_sgd(self, eta: float) -> None:
        """Fuse the descent step into later backward passes.  A bf16 net gets fp32 master weights on first
        use, initialised from the current bf16 weights."""
        if eta != 0.0 and self.dtype == "bf16" and self.master_w is None:
            self.master_w = [t.float() for t in self.w]
            self._check(lf_set_master_weights(self.handle, [t.data_ptr() for t in self.master_w]))
        self._check(lf_set_sgd(self.handle, eta))

    def forward(self) -> None:
        self._check(lf_forward(self.handle, self.x.data_ptr(), self._stream()))

    def backward(self, k: int = 1) -> None:
        self._check(lf_backward_leapfrog(self.handle, self.y.data_ptr(), k, self._stream()))

    def _view(self, ptr: int, shape, dtype):
        """A torch view of library-owned workspace memory (inside self.workspace)."""
        t = self.torch
        off = ptr - self.workspace.data_ptr()
        n = 1
        for s in shape:
            n *= s
        esz = t.empty(0, dtype=dtype).element_size()
        return self.workspace[off: off + n * esz].view(dtype).view(*shape)

    def activation(self, l: int):
        if l == 1:
            return self.x
        st, pa, _ = lf_activations(self.handle, l)
        self._check(st)
        return self._view(pa, (self.B, self.widths[l - 1]), self.tdtype)

    def delta(self, l: int):
        st, _, pd = lf_activations(self.handle, l)
        self._check(st)
        return self._view(pd, (self.B, self.widths[l - 1]), self.torch.float32)

    def grads(self, l: int):
        st, pw, pb = lf_grads(self.handle, l)
        self._check(st)
        assert pw == self.nabla_w[l - 2].data_ptr() and pb == self.nabla_b[l - 2].data_ptr()
        return self.nabla_w[l - 2], self.nabla_b[l - 2]

    def close(self) -> None:
        if self.handle is not None:
            lf_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
