"""ctypes binding of the C oracle (test infrastructure, not product code).

Every function converts numpy arrays to the layouts ``bcnn_oracle.c``
documents, calls it, and hands the result back.  No arithmetic happens here.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, name) for name in ("bcnn_oracle.c", "bcnn_branches_oracle.c", "bcnn_pool_oracle.c")]
_LIB = os.path.join(_HERE, "libbcnn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle's C files with gcc (-O3, OpenMP, baseline x86-64 so the
    library also runs on a host other than the one that built it)."""
    global _lib
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(p) for p in _SRCS)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
             "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp] + _SRCS + ["-lm"])
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
    lib.oracle_sign_bias_f32.argtypes = [vp, vp, i64, i64, i64, vp]
    lib.oracle_sign_bias_f32.restype = None
    lib.oracle_branches_real.argtypes = [vp] * 5 + [i32] * 8 + [vp]
    lib.oracle_branches_real.restype = i32
    lib.oracle_branches_pm1.argtypes = [vp, i32, vp, vp, vp, vp] + [i32] * 9 + [vp, vp, vp]
    lib.oracle_branches_pm1.restype = i32
    lib.oracle_module_epilogue.argtypes = [vp, vp, vp, vp, vp, i64, i32, vp, vp]
    lib.oracle_module_epilogue.restype = None
    lib.oracle_module_tail.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp]
    lib.oracle_module_tail.restype = None
    lib.oracle_store_f16.argtypes = [vp, i64, vp, vp]
    lib.oracle_store_f16.restype = None
    lib.oracle_store_bf16.argtypes = [vp, i64, vp, vp]
    lib.oracle_store_bf16.restype = None
    lib.oracle_load_bf16.argtypes = [vp, i64, vp]
    lib.oracle_load_bf16.restype = None
    lib.oracle_avgpool_nhwc.argtypes = [vp] + [i32] * 5 + [vp, vp]
    lib.oracle_avgpool_nhwc.restype = i32
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


def sign_bias_f32(x, bias):
    """x [outer, C, inner] float32, bias [C] float32 -> int8 +-1 of x's shape:
    sign(x + bias[c]) with the sum rounded to float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bias = np.ascontiguousarray(bias, dtype=np.float32)
    if x.ndim != 3 or bias.shape != (x.shape[1],):
        raise ValueError("x must be [outer, C, inner] and bias [C]")
    s = np.empty(x.shape, dtype=np.int8)
    _load().oracle_sign_bias_f32(_ptr(x), _ptr(bias), x.shape[0], x.shape[1], x.shape[2], _ptr(s))
    return s


def branches_real(a, b, w, g, h, stride=1, pad=0):
    """F x F binary convolution as F*F shifted 1x1 branches, from the real
    tensor.  a [N,C,H,W] float32, b [P,C] float32, w [O,C,F,F] +-1,
    g, h [P,O] float32 -> z [N,Ho,Wo,O] float64."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    w = _pm1(w, 4, "w")
    n, c, hh, ww = a.shape
    o, c2, f, f2 = w.shape
    p = f * f
    b = np.ascontiguousarray(b, dtype=np.float32)
    g = np.ascontiguousarray(g, dtype=np.float32)
    h = np.ascontiguousarray(h, dtype=np.float32)
    if c2 != c or f2 != f or b.shape != (p, c) or g.shape != (p, o) or h.shape != (p, o):
        raise ValueError("shape mismatch")
    lib = _load()
    ho, wo = lib.oracle_out_dim(hh, f, stride, pad), lib.oracle_out_dim(ww, f, stride, pad)
    z = np.empty((n, max(ho, 0), max(wo, 0), o), dtype=np.float64)
    rc = lib.oracle_branches_real(_ptr(a), _ptr(b), _ptr(w), _ptr(g), _ptr(h),
                                  n, c, hh, ww, o, f, stride, pad, _ptr(z))
    if rc != 0:
        raise ValueError("oracle_branches_real failed: %d" % rc)
    return z


def branches_pm1(xb, padv, w, g, h=None, stride=1, pad=0, taps=False):
    """The same on binarised operands.  xb [P,N,C,H,W] or [1,N,C,H,W] (shared by
    all branches) +-1, padv [P,C] from {-1,0,+1}, g [P,O] float32, h [O] float32
    or None.  w is [O,C,F,F] +-1 (shifted construction, P = F*F) or [O,C,P] (P
    parallel 1x1 branches, no shift).  Returns (z64, z32[, y_taps]) with
    z [N,Ho,Wo,O] and y_taps [N,Ho,Wo,O,P] int32."""
    xb = _pm1(xb, 5, "xb")
    w = np.ascontiguousarray(w, dtype=np.int8)
    bcount, n, c, hh, ww = xb.shape
    if w.ndim == 4:
        o, c2, f, f2 = w.shape
        p = f * f
    elif w.ndim == 3:
        o, c2, p = w.shape
        f = f2 = 1
    else:
        raise ValueError("w must be [O,C,F,F] or [O,C,P]")
    padv = np.ascontiguousarray(padv, dtype=np.int8)
    g = np.ascontiguousarray(g, dtype=np.float32)
    if h is not None:
        h = np.ascontiguousarray(h, dtype=np.float32)
    if c2 != c or f2 != f or bcount not in (1, p) or padv.shape != (p, c) or g.shape != (p, o) \
            or (h is not None and h.shape != (o,)):
        raise ValueError("shape mismatch")
    lib = _load()
    ho, wo = lib.oracle_out_dim(hh, f, stride, pad), lib.oracle_out_dim(ww, f, stride, pad)
    shape = (n, max(ho, 0), max(wo, 0), o)
    z64 = np.empty(shape, dtype=np.float64)
    z32 = np.empty(shape, dtype=np.float32)
    yt = np.empty(shape + (p,), dtype=np.int32) if taps else None
    shared = 1 if (bcount == 1 and p > 1) else 0
    rc = lib.oracle_branches_pm1(_ptr(xb), shared, _ptr(padv),
                                 _ptr(w), _ptr(g), _ptr(h) if h is not None else None,
                                 n, c, hh, ww, o, f, p, stride, pad, _ptr(z64), _ptr(z32),
                                 _ptr(yt) if taps else None)
    if rc != 0:
        raise ValueError("oracle_branches_pm1 failed: %d" % rc)
    return (z64, z32, yt) if taps else (z64, z32)


def module_epilogue(y, gamma, beta, identity=None, alpha=None):
    """Batch-norm scale and bias, identity addition, PReLU after a binary
    convolution.  y [..., O] int32, gamma/beta/alpha [O] float32, identity
    float32 of y's shape (or None) -> (r64, r32) of y's shape."""
    y = np.ascontiguousarray(y, dtype=np.int32)
    o = y.shape[-1]
    gamma = np.ascontiguousarray(gamma, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    if gamma.shape != (o,) or beta.shape != (o,):
        raise ValueError("gamma and beta must have one entry per output channel")
    if identity is not None:
        identity = np.ascontiguousarray(identity, dtype=np.float32)
        if identity.shape != y.shape:
            raise ValueError("identity must have the shape of y")
    if alpha is not None:
        alpha = np.ascontiguousarray(alpha, dtype=np.float32)
        if alpha.shape != (o,):
            raise ValueError("alpha must have one entry per output channel")
    r64 = np.empty(y.shape, dtype=np.float64)
    r32 = np.empty(y.shape, dtype=np.float32)
    _load().oracle_module_epilogue(_ptr(y), _ptr(gamma), _ptr(beta),
                                   _ptr(identity) if identity is not None else None,
                                   _ptr(alpha) if alpha is not None else None,
                                   y.size // o, o, _ptr(r64), _ptr(r32))
    return r64, r32


def module_tail(z64, z32, identity=None, alpha=None):
    """Identity addition and PReLU on a branch sum z (the tail of a module
    with parallel branches).  z64 float64 and z32 float32 of the same shape
    [..., O]; identity float32 of that shape or None; alpha [O] or None ->
    (r64, r32)."""
    z64 = np.ascontiguousarray(z64, dtype=np.float64)
    z32 = np.ascontiguousarray(z32, dtype=np.float32)
    if z64.shape != z32.shape:
        raise ValueError("z64 and z32 must have the same shape")
    o = z32.shape[-1]
    if identity is not None:
        identity = np.ascontiguousarray(identity, dtype=np.float32)
        if identity.shape != z32.shape:
            raise ValueError("identity must have the shape of z")
    if alpha is not None:
        alpha = np.ascontiguousarray(alpha, dtype=np.float32)
        if alpha.shape != (o,):
            raise ValueError("alpha must have one entry per output channel")
    r64 = np.empty(z64.shape, dtype=np.float64)
    r32 = np.empty(z32.shape, dtype=np.float32)
    _load().oracle_module_tail(_ptr(z64), _ptr(z32), _ptr(identity) if identity is not None else None,
                               _ptr(alpha) if alpha is not None else None, z32.size // o, o,
                               _ptr(r64), _ptr(r32))
    return r64, r32


def replicate_channels(x, r, axis=1):
    """Channel replication by an integer factor (paper, Section 4.2.2: a block
    that widens the network sees every real channel R times): the tensor with
    its channel axis repeated r times, channel k = j*C + c being a copy of
    channel c.  Here the copy is made for real (numpy.tile): the definition
    the library's bookkeeping is checked against."""
    x = np.asarray(x)
    if int(r) < 1:
        raise ValueError("replication factor must be >= 1")
    reps = [1] * x.ndim
    reps[axis] = int(r)
    return np.tile(x, reps)


def avgpool_nhwc(a, s):
    """S x S average pooling with stride S of a channel-last real map (paper,
    Section 4.2.3): a [N, H, W, C] float32 -> (p64, p32), both
    [N, H // s, W // s, C]: double sums, and the float chain in raster order."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != 4:
        raise ValueError("a must be [N, H, W, C]")
    n, h, w, c = a.shape
    s = int(s)
    if s < 1 or h // s < 1 or w // s < 1:
        raise ValueError("empty pooled map")
    p64 = np.empty((n, h // s, w // s, c), dtype=np.float64)
    p32 = np.empty((n, h // s, w // s, c), dtype=np.float32)
    rc = _load().oracle_avgpool_nhwc(_ptr(a), n, h, w, c, s, _ptr(p64), _ptr(p32))
    if rc != 0:
        raise ValueError("oracle_avgpool_nhwc failed: %d" % rc)
    return p64, p32


def store_f16(x):
    """float32 array -> the values as a binary16 stream stores them (numpy
    float16 array of the same shape; the oracle produces the bit patterns)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    code = np.empty(x.shape, dtype=np.uint16)
    _load().oracle_store_f16(_ptr(x), x.size, _ptr(code), None)
    return code.view(np.float16)


def store_bf16(x):
    """float32 array -> (uint16 bfloat16 patterns, the stored values as float32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    code = np.empty(x.shape, dtype=np.uint16)
    back = np.empty(x.shape, dtype=np.float32)
    _load().oracle_store_bf16(_ptr(x), x.size, _ptr(code), _ptr(back))
    return code, back


def load_bf16(code):
    """uint16 bfloat16 patterns -> float32 values."""
    code = np.ascontiguousarray(code, dtype=np.uint16)
    out = np.empty(code.shape, dtype=np.float32)
    _load().oracle_load_bf16(_ptr(code), code.size, _ptr(out))
    return out
