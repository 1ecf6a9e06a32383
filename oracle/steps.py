"""ctypes access to the plain-C oracle steps (cbinfer_oracle.c), one Python function per step.

TEST INFRASTRUCTURE ONLY (see the C file's header).  Arrays are planar float32 [C][H][W];
flags and maps are uint8 [H][W]; lists are int32, ascending.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cbinfer_oracle.c")
_LIB = os.path.join(_HERE, "libcbinfer_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = C.CDLL(build())
            f32p, u8p, i32p = C.POINTER(C.c_float), C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
            i, i64 = C.c_int, C.c_int64
            lib.orc_conv_dense.argtypes = [f32p, i, i, i, f32p, f32p, i, i, i, i, i, i, i, f32p]
            lib.orc_conv_dense.restype = None
            lib.orc_conv_update.argtypes = [f32p, i, i, i, f32p, f32p, i, i, i, i, i, i, i, i32p, i64, f32p]
            lib.orc_conv_update.restype = None
            lib.orc_maxpool.argtypes = [f32p, i, i, i, i, f32p]
            lib.orc_maxpool.restype = None
            lib.orc_detect.argtypes = [f32p, f32p, i, i64, C.c_float, u8p]
            lib.orc_detect.restype = i64
            lib.orc_update_ref.argtypes = [f32p, f32p, i, i64, u8p, i]
            lib.orc_update_ref.restype = None
            lib.orc_update_set.argtypes = [u8p, i, i, i, i, i, i, u8p]
            lib.orc_update_set.restype = None
            lib.orc_extract.argtypes = [u8p, i64, i32p]
            lib.orc_extract.restype = i64
            lib.orc_pool_set.argtypes = [u8p, i, i, i, u8p]
            lib.orc_pool_set.restype = None
            lib.orc_round_bf16.argtypes = [f32p, i64]
            lib.orc_round_bf16.restype = None
            lib.orc_max_threads.argtypes = []
            lib.orc_max_threads.restype = i
            _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint8))


def _conv_out_hw(H, W, kh, kw, s, p):
    return (H + 2 * p - kh) // s + 1, (W + 2 * p - kw) // s + 1


def conv_dense(x, w, b, stride=1, pad=0, relu=False, bf16=False):
    lib = _load()
    x, xp = _f32(x)
    w, wp = _f32(w)
    Cc, H, W = x.shape
    M, C2, kh, kw = w.shape
    assert C2 == Cc
    if b is None:
        b = np.zeros(M, np.float32)
    b, bp = _f32(b)
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    y = np.empty((M, Ho, Wo), np.float32)
    lib.orc_conv_dense(xp, Cc, H, W, wp, bp, M, kh, kw, stride, pad, int(relu), int(bf16),
                       y.ctypes.data_as(C.POINTER(C.c_float)))
    return y


def conv_update(x, w, b, upd_list, y, stride=1, pad=0, relu=False, bf16=False):
    """In place: recompute y at the listed output positions from x."""
    lib = _load()
    x, xp = _f32(x)
    w, wp = _f32(w)
    Cc, H, W = x.shape
    M, C2, kh, kw = w.shape
    assert C2 == Cc and y.dtype == np.float32 and y.flags.c_contiguous
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    assert y.shape == (M, Ho, Wo)
    if b is None:
        b = np.zeros(M, np.float32)
    b, bp = _f32(b)
    lst = np.ascontiguousarray(upd_list, dtype=np.int32)
    lib.orc_conv_update(xp, Cc, H, W, wp, bp, M, kh, kw, stride, pad, int(relu), int(bf16),
                        lst.ctypes.data_as(C.POINTER(C.c_int32)), lst.size,
                        y.ctypes.data_as(C.POINTER(C.c_float)))
    return y


def maxpool(x, k=2):
    lib = _load()
    x, xp = _f32(x)
    Cc, H, W = x.shape
    y = np.empty((Cc, H // k, W // k), np.float32)
    lib.orc_maxpool(xp, Cc, H, W, k, y.ctypes.data_as(C.POINTER(C.c_float)))
    return y


def detect(x, ref, tau):
    """uint8 [H][W] change flags."""
    lib = _load()
    x, xp = _f32(x)
    ref, rp = _f32(ref)
    assert x.shape == ref.shape
    Cc, H, W = x.shape
    flag = np.empty((H, W), np.uint8)
    lib.orc_detect(xp, rp, Cc, H * W, np.float32(tau), flag.ctypes.data_as(C.POINTER(C.c_uint8)))
    return flag


def update_ref(x, ref, flag, mode=0):
    """In place on ref."""
    lib = _load()
    x, xp = _f32(x)
    assert ref.dtype == np.float32 and ref.flags.c_contiguous and ref.shape == x.shape
    flag, fp = _u8(flag)
    Cc, H, W = x.shape
    lib.orc_update_ref(xp, ref.ctypes.data_as(C.POINTER(C.c_float)), Cc, H * W, fp, int(mode))
    return ref


def update_set(flag, kh, kw, stride=1, pad=0):
    lib = _load()
    flag, fp = _u8(flag)
    H, W = flag.shape
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    upd = np.empty((Ho, Wo), np.uint8)
    lib.orc_update_set(fp, H, W, kh, kw, stride, pad, upd.ctypes.data_as(C.POINTER(C.c_uint8)))
    return upd


def extract(map_):
    lib = _load()
    m, mp = _u8(map_)
    lst = np.empty(m.size, np.int32)
    n = lib.orc_extract(mp, m.size, lst.ctypes.data_as(C.POINTER(C.c_int32)))
    return lst[:n].copy()


def pool_set(upd, k=2):
    lib = _load()
    upd, up = _u8(upd)
    H, W = upd.shape
    out = np.empty((H // k, W // k), np.uint8)
    lib.orc_pool_set(up, H, W, k, out.ctypes.data_as(C.POINTER(C.c_uint8)))
    return out


def round_bf16(a):
    lib = _load()
    a = np.array(a, dtype=np.float32, copy=True, order="C")
    lib.orc_round_bf16(a.ctypes.data_as(C.POINTER(C.c_float)), a.size)
    return a


def max_threads() -> int:
    return int(_load().orc_max_threads())
