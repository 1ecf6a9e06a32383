"""ctypes binding of include/cbinfer.h.  Function names mirror the C ABI; this file marshals
arguments (numpy weights, torch device pointers, the current HIP stream) and nothing else.
There is no fallback: if the shared library is missing or no GPU is present, calls raise."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

OP_CONV, OP_MAXPOOL = 0, 1
F32, BF16 = 0, 1
FLAG_HOLD_REFERENCE = 1
FLAG_LISTS_EVERY_FRAME = 2
FLAG_PIPELINE_FRAMES = 4
LIST_CHANGED, LIST_UPDATE, LIST_POOLED = 0, 1, 2
MAP_REFERENCE, MAP_OUTPUT = 0, 1
STEP_NAMES = ["detect", "dilate", "compact", "gemm", "pool", "output"]

EXPORTS = [
    "cbinfer_workspace_bytes", "cbinfer_create", "cbinfer_process_frame", "cbinfer_reset",
    "cbinfer_destroy", "cbinfer_last_error", "cbinfer_set_mode", "cbinfer_layer_shape",
    "cbinfer_layer_counts", "cbinfer_read_list", "cbinfer_read_map", "cbinfer_set_profiling",
    "cbinfer_read_profile", "cbinfer_create_static", "cbinfer_static_workspace_bytes", "cbinfer_flush",
]


class cbinfer_layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("cin", C.c_int32), ("cout", C.c_int32), ("kh", C.c_int32),
                ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32), ("relu", C.c_int32),
                ("dense", C.c_int32), ("propagate", C.c_int32), ("threshold", C.c_float), ("weight", C.c_void_p),
                ("bias", C.POINTER(C.c_float))]


class cbinfer_network(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layers", C.POINTER(cbinfer_layer)), ("in_c", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("n_streams", C.c_int32), ("dtype", C.c_int32),
                ("flags", C.c_uint32), ("stream", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t)]


class CBInferError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("cbinfer error %d: %s" % (code, message))
        self.code = code


_lib = None


def library_path() -> str:
    """The in-tree build, or another build of the same library named by CBINFER_LIBRARY."""
    return os.environ.get("CBINFER_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                             "libcbinfer_hip.so")


def load_library():
    """Load libcbinfer_hip.so (built by paper_1704_04313_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(path + " is not built; run `python -m paper_1704_04313_amd.build`")
    # torch first: its wheel carries a HIP runtime of its own (same soname as the system's).  Loaded
    # first, it is the one this library binds to as well; loaded second, the process would hold two
    # runtimes and the later one finds no device.
    import torch  # noqa: F401
    lib = C.CDLL(path)
    st = C.c_void_p
    lib.cbinfer_workspace_bytes.argtypes = [C.POINTER(cbinfer_network)]
    lib.cbinfer_workspace_bytes.restype = C.c_size_t
    lib.cbinfer_create.argtypes = [C.POINTER(cbinfer_network), C.c_float]
    lib.cbinfer_create.restype = st
    lib.cbinfer_create_static.argtypes = [C.POINTER(cbinfer_network), C.c_float]
    lib.cbinfer_create_static.restype = st
    lib.cbinfer_static_workspace_bytes.argtypes = []
    lib.cbinfer_static_workspace_bytes.restype = C.c_size_t
    lib.cbinfer_process_frame.argtypes = [st, C.c_void_p, C.c_void_p]
    lib.cbinfer_process_frame.restype = C.c_int
    lib.cbinfer_flush.argtypes = [st]
    lib.cbinfer_flush.restype = C.c_int
    lib.cbinfer_reset.argtypes = [st]
    lib.cbinfer_reset.restype = C.c_int
    lib.cbinfer_destroy.argtypes = [st]
    lib.cbinfer_destroy.restype = None
    lib.cbinfer_last_error.argtypes = []
    lib.cbinfer_last_error.restype = C.c_char_p
    lib.cbinfer_set_mode.argtypes = [st, C.c_int]
    lib.cbinfer_set_mode.restype = C.c_int
    lib.cbinfer_layer_shape.argtypes = [st, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.cbinfer_layer_shape.restype = C.c_int
    lib.cbinfer_layer_counts.argtypes = [st, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.cbinfer_layer_counts.restype = C.c_int
    lib.cbinfer_read_list.argtypes = [st, C.c_int, C.c_int, C.POINTER(C.c_int32), C.c_int64, C.POINTER(C.c_int64)]
    lib.cbinfer_read_list.restype = C.c_int
    lib.cbinfer_read_map.argtypes = [st, C.c_int, C.c_int, C.POINTER(C.c_float), C.c_size_t]
    lib.cbinfer_read_map.restype = C.c_int
    lib.cbinfer_set_profiling.argtypes = [st, C.c_int]
    lib.cbinfer_set_profiling.restype = C.c_int
    lib.cbinfer_read_profile.argtypes = [st, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.cbinfer_read_profile.restype = C.c_int
    _lib = lib
    return lib


def _last_error(lib) -> str:
    return (lib.cbinfer_last_error() or b"").decode("utf-8", "replace")


def _describe(layers, params, in_shape, n_streams, flags, tau_per_layer, dense_layers, keep, dtype=F32,
              propagate_layers=()):
    """Build the C network description.  `keep` collects every numpy array the pointers refer to."""
    arr = (cbinfer_layer * len(layers))()
    for l, L in enumerate(layers):
        d = arr[l]
        if L.kind == "conv":
            w, b = params[l]
            w = np.ascontiguousarray(w, dtype=np.float32)
            assert w.shape == (L.cout, L.cin, L.kh, L.kw), "weight shape"
            keep.append(w)
            d.kind, d.cin, d.cout, d.kh, d.kw = OP_CONV, L.cin, L.cout, L.kh, L.kw
            d.stride, d.pad, d.relu = L.stride, L.pad, int(L.relu)
            d.dense = int(l in dense_layers)
            d.propagate = int(l in propagate_layers)
            d.threshold = -1.0 if tau_per_layer is None else float(tau_per_layer[l])
            d.weight = w.ctypes.data_as(C.c_void_p)
            if b is not None:
                b = np.ascontiguousarray(b, dtype=np.float32)
                keep.append(b)
                d.bias = b.ctypes.data_as(C.POINTER(C.c_float))
        else:
            d.kind, d.kh, d.kw, d.stride, d.pad = OP_MAXPOOL, L.kh, L.kw, L.stride, 0
            d.threshold = -1.0
    net = cbinfer_network()
    net.n_layers = len(layers)
    net.layers = arr
    net.in_c, net.in_h, net.in_w = (int(v) for v in in_shape)
    net.n_streams = int(n_streams)
    net.dtype = int(dtype)
    net.flags = int(flags)
    keep.append(arr)
    return net


def cbinfer_workspace_bytes(layers, params, in_shape, n_streams=1, flags=0, dtype=F32) -> int:
    lib = load_library()
    keep: list = []
    net = _describe(layers, params, in_shape, n_streams, flags, None, (), keep, dtype)
    n = lib.cbinfer_workspace_bytes(C.byref(net))
    if n == 0:
        raise CBInferError(-1, _last_error(lib))
    return int(n)


class CBInfer:
    """One cbinfer_state.  Frames and outputs are torch CUDA tensors (device memory only);
    all work is enqueued on the torch stream that was current at construction."""

    def __init__(self, layers, params, in_shape, tau, *, n_streams: int = 1, hold_reference: bool = False,
                 dense_layers: Sequence[int] = (), caller_workspace: bool = True, dtype: int = F32,
                 propagate_layers: Sequence[int] = (), lists_every_frame: bool = False,
                 static_workspace: bool = False, pipeline_frames: bool = False):
        import torch
        self._torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise CBInferError(-4, "no GPU visible to torch; the HIP path has no CPU fallback")
        self.layers = list(layers)
        self.n_streams = int(n_streams)
        self.in_shape = tuple(int(v) for v in in_shape)
        per_layer = None if np.isscalar(tau) else [(-1.0 if t is None else float(t)) for t in tau]
        global_tau = float(tau) if np.isscalar(tau) else 0.0
        keep: list = []
        flags = ((FLAG_HOLD_REFERENCE if hold_reference else 0) | (FLAG_LISTS_EVERY_FRAME if lists_every_frame else 0) |
                 (FLAG_PIPELINE_FRAMES if pipeline_frames else 0))
        self.dtype = int(dtype)
        net = _describe(self.layers, params, self.in_shape, n_streams, flags, per_layer, set(dense_layers), keep,
                        self.dtype, set(propagate_layers))
        self.stream = torch.cuda.current_stream()
        net.stream = C.c_void_p(self.stream.cuda_stream)
        self.workspace = None
        if caller_workspace and not static_workspace:
            nbytes = self.lib.cbinfer_workspace_bytes(C.byref(net))
            if nbytes == 0:
                raise CBInferError(-1, _last_error(self.lib))
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
            ptr = (self.workspace.data_ptr() + 255) // 256 * 256
            net.workspace = C.c_void_p(ptr)
            net.workspace_bytes = nbytes
        create = self.lib.cbinfer_create_static if static_workspace else self.lib.cbinfer_create
        self._state = create(C.byref(net), C.c_float(global_tau))
        if not self._state:
            raise CBInferError(-1, _last_error(self.lib))
        c, h, w = self.layer_shape(len(self.layers) - 1)
        self.out_shape = (self.n_streams, c, h, w)

    # -- C ABI calls, same names --------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise CBInferError(rc, _last_error(self.lib))

    def process_frame(self, frame, out=None):
        """frame: float32 CUDA tensor [n_streams][C][H][W] (or [C][H][W] for one stream)."""
        torch = self._torch
        assert frame.is_cuda and frame.dtype == torch.float32 and frame.is_contiguous()
        assert frame.numel() == self.n_streams * int(np.prod(self.in_shape)), "frame size"
        if out is None:
            out = torch.empty(self.out_shape, dtype=torch.float32, device=frame.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert out.numel() == int(np.prod(self.out_shape))
        self._check(self.lib.cbinfer_process_frame(self._state, C.c_void_p(frame.data_ptr()),
                                                   C.c_void_p(out.data_ptr())))
        return out

    def process_frame_ptr(self, frame_ptr: int, out_ptr: int):
        """Same call with raw device addresses (no tensor checks)."""
        rc = self.lib.cbinfer_process_frame(self._state, frame_ptr, out_ptr)
        if rc != 0:
            raise CBInferError(rc, _last_error(self.lib))

    def flush(self):
        self._check(self.lib.cbinfer_flush(self._state))

    def reset(self):
        self._check(self.lib.cbinfer_reset(self._state))

    def set_mode(self, force_dense: bool):
        self._check(self.lib.cbinfer_set_mode(self._state, int(bool(force_dense))))

    def layer_shape(self, layer: int):
        c, h, w = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self.lib.cbinfer_layer_shape(self._state, layer, C.byref(c), C.byref(h), C.byref(w)))
        return c.value, h.value, w.value

    def layer_counts(self, layer: int):
        a, b = C.c_int64(), C.c_int64()
        self._check(self.lib.cbinfer_layer_counts(self._state, layer, C.byref(a), C.byref(b)))
        return a.value, b.value

    def read_list(self, layer: int, which: int) -> np.ndarray:
        n = C.c_int64()
        self._check(self.lib.cbinfer_read_list(self._state, layer, which, None, 0, C.byref(n)))
        buf = np.empty(max(n.value, 1), np.int32)
        self._check(self.lib.cbinfer_read_list(self._state, layer, which,
                                               buf.ctypes.data_as(C.POINTER(C.c_int32)), n.value, C.byref(n)))
        return buf[:n.value].copy()

    def read_map(self, layer: int, which: int) -> np.ndarray:
        L = self.layers[layer]
        if which == MAP_OUTPUT:
            c, h, w = self.layer_shape(layer)
        else:
            if layer == 0:
                c, h, w = self.in_shape
            else:
                c, h, w = self.layer_shape(layer - 1)
        buf = np.empty((self.n_streams, c, h, w), np.float32)
        self._check(self.lib.cbinfer_read_map(self._state, layer, which,
                                              buf.ctypes.data_as(C.POINTER(C.c_float)), buf.size))
        return buf

    def set_profiling(self, enable: bool):
        self._check(self.lib.cbinfer_set_profiling(self._state, int(bool(enable))))

    def read_profile(self, layer: int, step: int):
        ms, n = C.c_double(), C.c_int64()
        self._check(self.lib.cbinfer_read_profile(self._state, layer, step, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def destroy(self):
        if getattr(self, "_state", None):
            self.lib.cbinfer_destroy(self._state)
            self._state = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
