"""ctypes binding of the C oracle (test infrastructure, not product code).

Every function converts numpy arrays to the layouts ``bcnn_oracle.c``
documents, calls it, and hands the result back.  No arithmetic happens here.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcnn_oracle.c")
_LIB = os.path.join(_HERE, "libbcnn_oracle.so")
_lib = None


def build(force=False):
    """Compile bcnn_oracle.c with gcc (-O3, OpenMP, baseline x86-64 so the
    library also runs on a host other than the one that built it)."""
    global _lib
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
             "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i32, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    lib.oracle_num_threads.restype = i32
    lib.oracle_out_dim.argtypes = [i32] * 4
    lib.oracle_out_dim.restype = i32
    lib.oracle_sign_f32.argtypes = [vp, i64, vp]
    lib.oracle_sign_f32.restype = None
    lib.oracle_conv2d_pm1.argtypes = [vp, vp] + [i32] * 9 + [vp]
    lib.oracle_conv2d_pm1.restype = i32
    lib.oracle_conv2d_pm1_at.argtypes = [vp, vp] + [i32] * 9 + [vp, i64, vp]
    lib.oracle_conv2d_pm1_at.restype = i32
    lib.oracle_threshold_sign.argtypes = [vp, vp, i64, i32, vp]
    lib.oracle_threshold_sign.restype = None
    lib.oracle_pack_channels.argtypes = [vp, i64, i64, i64, vp]
    lib.oracle_pack_channels.restype = None
    lib.oracle_unpack_channels.argtypes = [vp, i64, i64, i64, vp]
    lib.oracle_unpack_channels.restype = None
    _lib = lib
    return lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _pm1(a, ndim, name):
    a = np.ascontiguousarray(a, dtype=np.int8)
    if a.ndim != ndim:
        raise ValueError("%s must have %d dimensions" % (name, ndim))
    return a


def num_threads():
    return int(_load().oracle_num_threads())


def out_dim(size, k, stride, pad):
    return int(_load().oracle_out_dim(size, k, stride, pad))


def sign_f32(x):
    """float32 array -> int8 array of +-1, same shape."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    s = np.empty(x.shape, dtype=np.int8)
    _load().oracle_sign_f32(_ptr(x), x.size, _ptr(s))
    return s


def conv2d_pm1(x, w, stride=1, pad=0):
    """x [N,C,H,W] +-1, w [O,C,KH,KW] +-1 -> y [N,Ho,Wo,O] int32."""
    x = _pm1(x, 4, "x")
    w = _pm1(w, 4, "w")
    n, c, h, wd = x.shape
    o, c2, kh, kw = w.shape
    if c2 != c:
        raise ValueError("channel mismatch")
    lib = _load()
    ho, wo = lib.oracle_out_dim(h, kh, stride, pad), lib.oracle_out_dim(wd, kw, stride, pad)
    y = np.empty((n, max(ho, 0), max(wo, 0), o), dtype=np.int32)
    rc = lib.oracle_conv2d_pm1(_ptr(x), _ptr(w), n, c, h, wd, o, kh, kw, stride, pad, _ptr(y))
    if rc != 0:
        raise ValueError("oracle_conv2d_pm1 failed: %d" % rc)
    return y


def conv2d_pm1_at(x, w, idx, stride=1, pad=0):
    """Single outputs: idx [count,4] of (n, oh, ow, o) -> int32 [count]."""
    x = _pm1(x, 4, "x")
    w = _pm1(w, 4, "w")
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    n, c, h, wd = x.shape
    o, c2, kh, kw = w.shape
    if c2 != c:
        raise ValueError("channel mismatch")
    out = np.empty(idx.shape[0], dtype=np.int32)
    rc = _load().oracle_conv2d_pm1_at(_ptr(x), _ptr(w), n, c, h, wd, o, kh, kw, stride, pad,
                                      _ptr(idx), idx.shape[0], _ptr(out))
    if rc != 0:
        raise ValueError("oracle_conv2d_pm1_at failed: %d" % rc)
    return out


def threshold_sign(y, thr):
    """y [..., O] int32, thr [O] int32 -> int8 +-1 of y's shape."""
    y = np.ascontiguousarray(y, dtype=np.int32)
    thr = np.ascontiguousarray(thr, dtype=np.int32)
    o = y.shape[-1]
    if thr.shape != (o,):
        raise ValueError("thr must have one entry per output channel")
    s = np.empty(y.shape, dtype=np.int8)
    _load().oracle_threshold_sign(_ptr(y), _ptr(thr), y.size // o, o, _ptr(s))
    return s


def pack_channels(s):
    """s [outer, C, inner] +-1 -> uint32 [outer, inner, ceil(C/32)]."""
    s = _pm1(s, 3, "s")
    outer, c, inner = s.shape
    dst = np.empty((outer, inner, (c + 31) // 32), dtype=np.uint32)
    _load().oracle_pack_channels(_ptr(s), outer, c, inner, _ptr(dst))
    return dst


def unpack_channels(p, channels):
    """uint32 [outer, inner, ceil(C/32)] -> int8 +-1 [outer, C, inner]."""
    p = np.ascontiguousarray(p, dtype=np.uint32)
    if p.ndim != 3 or p.shape[2] != (channels + 31) // 32:
        raise ValueError("packed array has the wrong shape")
    outer, inner, _ = p.shape
    s = np.empty((outer, channels, inner), dtype=np.int8)
    _load().oracle_unpack_channels(_ptr(p), outer, channels, inner, _ptr(s))
    return s
