"""Argument marshalling between Python and libfdg.so.  No arithmetic happens here: torch only owns
device memory and streams; every step of the module's forward, delayed backward and update runs in
the library's kernels.  Function names and argument order follow include/fdg.h and include/fdg_chain.h."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfdg.so")

STATUS_NAMES = {0: "FDG_OK", 1: "FDG_ERR_INVALID_ARG", 2: "FDG_ERR_UNSUPPORTED", 3: "FDG_ERR_WORKSPACE_TOO_SMALL",
                4: "FDG_ERR_QUEUE_FULL", 5: "FDG_ERR_QUEUE_EMPTY", 6: "FDG_ERR_NO_GRAD", 7: "FDG_ERR_HIP"}
FDG_OK, FDG_ERR_INVALID_ARG, FDG_ERR_UNSUPPORTED, FDG_ERR_WORKSPACE_TOO_SMALL = 0, 1, 2, 3
FDG_ERR_QUEUE_FULL, FDG_ERR_QUEUE_EMPTY, FDG_ERR_NO_GRAD, FDG_ERR_HIP = 4, 5, 6, 7


class FdgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")


class fdg_layer_desc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32), ("stride", ctypes.c_int32)]


class fdg_profile_entry(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("kernel", ctypes.c_char * 80), ("calls", ctypes.c_int64), ("total_ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


class fdg_module_desc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("c_in", ctypes.c_int32), ("h_in", ctypes.c_int32), ("w_in", ctypes.c_int32),
                ("num_layers", ctypes.c_int32), ("layers", ctypes.POINTER(fdg_layer_desc)),
                ("delay", ctypes.c_int32), ("is_bottom", ctypes.c_int32), ("num_classes", ctypes.c_int32),
                ("beta", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("bn_eps", ctypes.c_float), ("bn_momentum", ctypes.c_float)]


_lib: Optional[ctypes.CDLL] = None

EXPORTS = ["fdg_module_workspace_bytes", "fdg_module_create", "fdg_module_workspace_bytes_ex", "fdg_module_create_ex", "fdg_lr_schedule", "fdg_forward", "fdg_backward_delayed", "fdg_update",
           "fdg_destroy", "fdg_param_count", "fdg_set_params", "fdg_get_params", "fdg_get_grads", "fdg_get_momentum",
           "fdg_bn_stat_count", "fdg_get_bn_running", "fdg_output_shape", "fdg_queue_state", "fdg_status_string",
           "fdg_profile_enable", "fdg_profile_read", "fdg_input_shape", "fdg_module_traits",
           "fdg_saved_read", "fdg_trace_bytes", "fdg_trace_attach", "fdg_trace_read", "fdg_overlap_enable",
           "fdg_chain_mailbox_bytes", "fdg_chain_create", "fdg_chain_step", "fdg_chain_state", "fdg_chain_destroy"]


def load() -> ctypes.CDLL:
    """Load libfdg.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_1906_09108_amd.build` "
                                "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    dp = ctypes.POINTER(fdg_module_desc)
    lib.fdg_module_workspace_bytes.argtypes, lib.fdg_module_workspace_bytes.restype = [dp], sz
    lib.fdg_module_create.argtypes, lib.fdg_module_create.restype = [dp, vp, sz, vp, ctypes.POINTER(vp)], i32
    lib.fdg_lr_schedule.argtypes, lib.fdg_lr_schedule.restype = [i32, i32], ctypes.c_float
    lib.fdg_module_workspace_bytes_ex.argtypes, lib.fdg_module_workspace_bytes_ex.restype = [dp, i32], sz
    lib.fdg_module_create_ex.argtypes, lib.fdg_module_create_ex.restype = [dp, i32, vp, sz, vp, ctypes.POINTER(vp)], i32
    lib.fdg_forward.argtypes, lib.fdg_forward.restype = [vp, vp, vp, vp, vp], i32
    lib.fdg_backward_delayed.argtypes, lib.fdg_backward_delayed.restype = [vp, vp, vp, vp], i32
    lib.fdg_update.argtypes, lib.fdg_update.restype = [vp, f32, vp], i32
    lib.fdg_destroy.argtypes, lib.fdg_destroy.restype = [vp], None
    lib.fdg_param_count.argtypes, lib.fdg_param_count.restype = [vp], sz
    for name in ("fdg_set_params", "fdg_get_params", "fdg_get_grads", "fdg_get_momentum", "fdg_get_bn_running"):
        getattr(lib, name).argtypes, getattr(lib, name).restype = [vp, vp, sz], i32
    lib.fdg_bn_stat_count.argtypes, lib.fdg_bn_stat_count.restype = [vp], sz
    lib.fdg_output_shape.argtypes, lib.fdg_output_shape.restype = [vp, ctypes.POINTER(i32 * 4)], i32
    lib.fdg_queue_state.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
    lib.fdg_queue_state.restype = i32
    lib.fdg_status_string.argtypes, lib.fdg_status_string.restype = [i32], ctypes.c_char_p
    lib.fdg_profile_enable.argtypes, lib.fdg_profile_enable.restype = [vp, i32], i32
    lib.fdg_overlap_enable.argtypes, lib.fdg_overlap_enable.restype = [vp, i32], i32
    lib.fdg_profile_read.argtypes = [vp, ctypes.POINTER(fdg_profile_entry), i32, ctypes.POINTER(i32)]
    lib.fdg_profile_read.restype = i32
    lib.fdg_input_shape.argtypes, lib.fdg_input_shape.restype = [vp, ctypes.POINTER(i32 * 4)], i32
    lib.fdg_module_traits.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.fdg_module_traits.restype = i32
    lib.fdg_saved_read.argtypes = [vp, ctypes.c_int64, i32, i32, vp, sz, ctypes.POINTER(i32 * 4)]
    lib.fdg_saved_read.restype = i32
    lib.fdg_trace_bytes.argtypes, lib.fdg_trace_bytes.restype = [vp], sz
    lib.fdg_trace_attach.argtypes, lib.fdg_trace_attach.restype = [vp, vp, sz], i32
    lib.fdg_trace_read.argtypes = [vp, i32, i32, vp, sz, ctypes.POINTER(i32 * 4), ctypes.POINTER(i32)]
    lib.fdg_trace_read.restype = i32
    lib.fdg_chain_mailbox_bytes.argtypes, lib.fdg_chain_mailbox_bytes.restype = [ctypes.POINTER(vp), i32], sz
    lib.fdg_chain_create.argtypes, lib.fdg_chain_create.restype = [ctypes.POINTER(vp), i32, vp, sz, ctypes.POINTER(vp)], i32
    lib.fdg_chain_step.argtypes, lib.fdg_chain_step.restype = [vp, vp, vp, f32, vp, ctypes.POINTER(i32), vp], i32
    lib.fdg_chain_state.argtypes = [vp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.fdg_chain_state.restype = i32
    lib.fdg_chain_destroy.argtypes, lib.fdg_chain_destroy.restype = [vp], None
    _lib = lib
    return lib


def make_desc(spec) -> Tuple[fdg_module_desc, object]:
    """C descriptor from any object with the descriptor's fields (e.g. fdg_workloads.ModuleSpec).
    Returns (desc, keepalive)."""
    arr = (fdg_layer_desc * len(spec.layers))()
    for i, L in enumerate(spec.layers):
        arr[i] = fdg_layer_desc(int(L.kind), int(L.c_in), int(L.c_out), int(L.stride))
    d = fdg_module_desc(int(spec.n), int(spec.c_in), int(spec.h_in), int(spec.w_in), len(spec.layers),
                        ctypes.cast(arr, ctypes.POINTER(fdg_layer_desc)), int(spec.delay), int(bool(spec.is_bottom)),
                        int(spec.num_classes), float(spec.beta), float(spec.momentum), float(spec.weight_decay),
                        float(spec.bn_eps), float(spec.bn_momentum))
    return d, arr


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = int(stream.cuda_stream)
    return h if h else None


# ---- the C entry points, same names, torch tensors in place of raw pointers ---------------------
def fdg_module_workspace_bytes(spec) -> int:
    d, keep = make_desc(spec)
    return int(load().fdg_module_workspace_bytes(ctypes.byref(d)))


def fdg_module_create(spec, workspace, stream=None) -> int:
    """workspace: a torch uint8 CUDA tensor of at least fdg_module_workspace_bytes(spec) bytes,
    256-byte aligned.  Returns the opaque module handle."""
    d, keep = make_desc(spec)
    out = ctypes.c_void_p()
    st = load().fdg_module_create(ctypes.byref(d), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                  _stream_handle(stream), ctypes.byref(out))
    if st != FDG_OK:
        raise FdgError(st, "fdg_module_create")
    return out.value


FDG_SAVE_ACTIVATIONS, FDG_SAVE_INPUT_AND_REPLAY, FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS = 0, 1, 2


def fdg_lr_schedule(epoch: int, warmup_epochs: int = 0) -> float:
    return float(load().fdg_lr_schedule(int(epoch), int(warmup_epochs)))


def fdg_module_workspace_bytes_ex(spec, save_mode: int) -> int:
    d, keep = make_desc(spec)
    return int(load().fdg_module_workspace_bytes_ex(ctypes.byref(d), int(save_mode)))


def fdg_module_create_ex(spec, save_mode: int, workspace, stream=None) -> int:
    d, keep = make_desc(spec)
    out = ctypes.c_void_p()
    st = load().fdg_module_create_ex(ctypes.byref(d), int(save_mode), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream_handle(stream), ctypes.byref(out))
    if st != FDG_OK:
        raise FdgError(st, "fdg_module_create_ex")
    return out.value


def _shape(handle: int, which: str) -> Tuple[int, int, int, int]:
    shp = (ctypes.c_int32 * 4)()
    getattr(load(), which)(handle, ctypes.byref(shp))
    return tuple(int(v) for v in shp)


def _dense(t, dtype_name: str, numel: int) -> bool:
    """The library reads raw pointers: a tensor handed to it must be what the header says it is (device memory,
    dense, of the stated element type and size), or the kernels would read out of bounds."""
    import torch
    return (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == getattr(torch, dtype_name)
            and t.numel() == numel)


def fdg_forward(handle: int, x, labels, y, stream=None) -> int:
    """FDG_ERR_INVALID_ARG without calling the library if a tensor is not a dense CUDA tensor of the type and size
    include/fdg.h states (x, y: float32; labels: int32 [n])."""
    n, c, h, w = _shape(handle, "fdg_input_shape")
    on, oc, oh, ow = _shape(handle, "fdg_output_shape")
    if x is None or y is None or not _dense(x, "float32", n * c * h * w) or not _dense(y, "float32", on * oc * oh * ow):
        return FDG_ERR_INVALID_ARG
    if labels is not None and not _dense(labels, "int32", n):
        return FDG_ERR_INVALID_ARG
    return int(load().fdg_forward(handle, _ptr(x), _ptr(labels), _ptr(y), _stream_handle(stream)))


def fdg_backward_delayed(handle: int, grad_out, grad_in, stream=None) -> int:
    """FDG_ERR_INVALID_ARG without calling the library if a tensor is not a dense float32 CUDA tensor of the forward's
    output (grad_out) or input (grad_in) size."""
    n, c, h, w = _shape(handle, "fdg_input_shape")
    on, oc, oh, ow = _shape(handle, "fdg_output_shape")
    if grad_out is not None and not _dense(grad_out, "float32", on * oc * oh * ow):
        return FDG_ERR_INVALID_ARG
    if grad_in is not None and not _dense(grad_in, "float32", n * c * h * w):
        return FDG_ERR_INVALID_ARG
    return int(load().fdg_backward_delayed(handle, _ptr(grad_out), _ptr(grad_in), _stream_handle(stream)))


def fdg_update(handle: int, lr: float, stream=None) -> int:
    return int(load().fdg_update(handle, float(lr), _stream_handle(stream)))


def fdg_destroy(handle: Optional[int]) -> None:
    if handle:
        load().fdg_destroy(handle)


class FdgModule:
    """Owns the workspace tensor and the handle of one module; every method is one C call."""

    def __init__(self, spec, device="cuda:0", stream=None, save_mode=FDG_SAVE_ACTIVATIONS):
        import torch
        self.torch = torch
        self.spec = spec
        self.device = torch.device(device)
        self.save_mode = int(save_mode)
        nbytes = fdg_module_workspace_bytes_ex(spec, self.save_mode)
        if nbytes == 0:
            raise FdgError(FDG_ERR_UNSUPPORTED, "fdg_module_workspace_bytes")
        self.workspace_bytes = nbytes
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        off = (-self.workspace.data_ptr()) % 256
        self._ws_view = self.workspace[off:off + nbytes]
        self.handle = fdg_module_create_ex(spec, self.save_mode, self._ws_view, stream)
        shp = (ctypes.c_int32 * 4)()
        load().fdg_output_shape(self.handle, ctypes.byref(shp))
        self.out_shape = tuple(int(v) for v in shp)
        self.is_top = bool(spec.layers) and int(spec.layers[-1].kind) in (3, 4)

    def close(self):
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize(self.device)
            fdg_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- hot path ----------------------------------------------------------------------------------
    def new_output(self):
        t = self.torch
        if self.is_top:
            return t.empty(self.out_shape[3], dtype=t.float32, device=self.device)
        return t.empty(self.out_shape, dtype=t.float32, device=self.device)

    def forward(self, x, labels=None, y=None, stream=None, check=True):
        if y is None:
            y = self.new_output()
        st = fdg_forward(self.handle, x, labels, y, stream)
        if check and st != FDG_OK:
            raise FdgError(st, "fdg_forward")
        return y if check else (st, y)

    def backward_delayed(self, grad_out=None, grad_in=None, stream=None, check=True):
        st = fdg_backward_delayed(self.handle, grad_out, grad_in, stream)
        if check and st != FDG_OK:
            raise FdgError(st, "fdg_backward_delayed")
        return grad_in if check else st

    def update(self, lr, stream=None, check=True):
        st = fdg_update(self.handle, lr, stream)
        if check and st != FDG_OK:
            raise FdgError(st, "fdg_update")
        return st

    # -- host accessors ----------------------------------------------------------------------------
    def param_count(self) -> int:
        return int(load().fdg_param_count(self.handle))

    def set_params(self, flat: np.ndarray) -> None:
        a = np.ascontiguousarray(flat, np.float32)
        st = load().fdg_set_params(self.handle, a.ctypes.data, a.size)
        if st != FDG_OK:
            raise FdgError(st, "fdg_set_params")

    def _get(self, name: str, count: int) -> np.ndarray:
        a = np.empty(count, np.float32)
        st = getattr(load(), name)(self.handle, a.ctypes.data, a.size)
        if st != FDG_OK:
            raise FdgError(st, name)
        return a

    def get_params(self):
        return self._get("fdg_get_params", self.param_count())

    def get_grads(self):
        return self._get("fdg_get_grads", self.param_count())

    def get_momentum(self):
        return self._get("fdg_get_momentum", self.param_count())

    def get_bn_running(self):
        return self._get("fdg_get_bn_running", int(load().fdg_bn_stat_count(self.handle)))

    def profile_enable(self, enable: bool) -> None:
        st = load().fdg_profile_enable(self.handle, int(bool(enable)))
        if st != FDG_OK:
            raise FdgError(st, "fdg_profile_enable")

    def overlap_enable(self, enable: bool) -> None:
        st = load().fdg_overlap_enable(self.handle, int(bool(enable)))
        if st != FDG_OK:
            raise FdgError(st, "fdg_overlap_enable")

    def profile_read(self) -> list:
        """[dict(name, kernel, calls, total_ms, flops, bytes)]: one entry per kernel class and, for
        convolutions, per kernel and layer shape, summed over the records since the enable."""
        n = ctypes.c_int32()
        st = load().fdg_profile_read(self.handle, None, 0, ctypes.byref(n))
        if st != FDG_OK:
            raise FdgError(st, "fdg_profile_read")
        cap = max(int(n.value), 1)
        arr = (fdg_profile_entry * cap)()
        st = load().fdg_profile_read(self.handle, arr, cap, ctypes.byref(n))
        if st != FDG_OK:
            raise FdgError(st, "fdg_profile_read")
        return [dict(name=arr[i].name.decode(), kernel=arr[i].kernel.decode(), calls=int(arr[i].calls),
                     total_ms=float(arr[i].total_ms), flops=float(arr[i].flops), bytes=float(arr[i].bytes))
                for i in range(min(n.value, cap))]

    # -- parity accessors (include/fdg.h): one C call each; the first call with a one-element buffer only asks for the shape
    def saved_read(self, seq: int, layer: int, which: int) -> np.ndarray:
        """A tensor of the saved forward `seq` as host float32 NCHW."""
        shp = (ctypes.c_int32 * 4)()
        probe = np.empty(1, np.float32)
        load().fdg_saved_read(self.handle, int(seq), int(layer), int(which), probe.ctypes.data, 0, ctypes.byref(shp))
        shape = tuple(int(v) for v in shp)
        if min(shape) <= 0:
            raise FdgError(FDG_ERR_INVALID_ARG, f"fdg_saved_read(seq={seq}, layer={layer}, which={which})")
        out = np.empty(shape, np.float32)
        st = load().fdg_saved_read(self.handle, int(seq), int(layer), int(which), out.ctypes.data, out.size, ctypes.byref(shp))
        if st != FDG_OK:
            raise FdgError(st, f"fdg_saved_read(seq={seq}, layer={layer}, which={which})")
        return out

    def trace_attach(self) -> None:
        """Allocates a trace buffer (torch owns the memory) and attaches it."""
        t = self.torch
        nbytes = int(load().fdg_trace_bytes(self.handle))
        self._trace = t.empty(nbytes + 256, dtype=t.uint8, device=self.device)
        off = (-self._trace.data_ptr()) % 256
        st = load().fdg_trace_attach(self.handle, int(self._trace.data_ptr()) + off, nbytes)
        if st != FDG_OK:
            raise FdgError(st, "fdg_trace_attach")

    def trace_detach(self) -> None:
        st = load().fdg_trace_attach(self.handle, None, 0)
        if st != FDG_OK:
            raise FdgError(st, "fdg_trace_attach")
        self._trace = None

    def trace_read(self, direction: int, layer: int) -> Tuple[np.ndarray, bool]:
        """(tensor as host float32 NCHW, already gated by the layer below)."""
        shp, gated = (ctypes.c_int32 * 4)(), ctypes.c_int32()
        probe = np.empty(1, np.float32)
        load().fdg_trace_read(self.handle, int(direction), int(layer), probe.ctypes.data, 0, ctypes.byref(shp), ctypes.byref(gated))
        shape = tuple(int(v) for v in shp)
        if min(shape) <= 0:
            raise FdgError(FDG_ERR_INVALID_ARG, f"fdg_trace_read(dir={direction}, layer={layer})")
        out = np.empty(shape, np.float32)
        st = load().fdg_trace_read(self.handle, int(direction), int(layer), out.ctypes.data, out.size, ctypes.byref(shp),
                                   ctypes.byref(gated))
        if st != FDG_OK:
            raise FdgError(st, f"fdg_trace_read(dir={direction}, layer={layer})")
        return out, bool(gated.value)

    def queue_state(self) -> Tuple[int, int, int]:
        o, a, b = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int64()
        load().fdg_queue_state(self.handle, ctypes.byref(o), ctypes.byref(a), ctypes.byref(b))
        return int(o.value), int(a.value), int(b.value)


class FdgChain:
    """K modules run as Algorithm I (include/fdg_chain.h).  Owns the modules' workspaces, the mailbox memory and
    the chain handle; step() is one C call."""

    def __init__(self, specs: Sequence, device="cuda:0", save_mode=FDG_SAVE_ACTIVATIONS):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.modules = [FdgModule(sp, device, save_mode=save_mode) for sp in specs]
        self.K = len(self.modules)
        self._handles = (ctypes.c_void_p * self.K)(*[m.handle for m in self.modules])
        nbytes = int(load().fdg_chain_mailbox_bytes(self._handles, self.K))
        if nbytes == 0 and self.K > 1:
            raise FdgError(FDG_ERR_INVALID_ARG, "fdg_chain_mailbox_bytes")
        self.mailbox = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        off = (-self.mailbox.data_ptr()) % 256
        self._mb_view = self.mailbox[off:off + max(nbytes, 1)]
        out = ctypes.c_void_p()
        st = load().fdg_chain_create(self._handles, self.K, _ptr(self._mb_view), nbytes, ctypes.byref(out))
        if st != FDG_OK:
            raise FdgError(st, "fdg_chain_create")
        self.handle = out.value
        top = self.modules[-1]
        self.top_y = top.new_output()

    def step(self, x, labels, lr: float, stream=None) -> int:
        """One iteration on batch (x, labels), both CUDA tensors.  Returns the 1-based batch whose loss and logits
        are now being written to self.top_y (0 while the last module idles)."""
        n, c, h, w = _shape(self.modules[0].handle, "fdg_input_shape")
        if not _dense(x, "float32", n * c * h * w) or not _dense(labels, "int32", n):
            raise FdgError(FDG_ERR_INVALID_ARG, "fdg_chain_step (x: dense float32 CUDA [n,c,h,w]; labels: int32 CUDA [n])")
        b = ctypes.c_int32()
        st = load().fdg_chain_step(self.handle, _ptr(x), _ptr(labels), float(lr), _ptr(self.top_y), ctypes.byref(b),
                                   _stream_handle(stream))
        if st != FDG_OK:
            raise FdgError(st, "fdg_chain_step")
        return int(b.value)

    def state(self) -> Tuple[int, list, list]:
        t = ctypes.c_int64()
        f, b = (ctypes.c_int32 * self.K)(), (ctypes.c_int32 * self.K)()
        load().fdg_chain_state(self.handle, ctypes.byref(t), f, b)
        return int(t.value), list(f), list(b)

    def close(self):
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize(self.device)
            load().fdg_chain_destroy(self.handle)
            self.handle = None
        for m in getattr(self, "modules", []):
            m.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
