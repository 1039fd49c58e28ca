"""ctypes binding of libbcnn.so: the C ABI of include/bcnn.h under the same names.

Argument marshalling only.  torch supplies device memory and the stream; every
step of the computation runs in the library's HIP kernels.  There is no CPU or
PyTorch fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbcnn.so")

BCNN_OK = 0
BCNN_ERR_INVALID_ARG = -1
BCNN_ERR_UNSUPPORTED = -2
BCNN_ERR_ALIGNMENT = -3
BCNN_ERR_DEVICE = -4

BCNN_F32, BCNN_F16, BCNN_I8, BCNN_BF16 = 0, 1, 2, 3
BCNN_VARIANT_AUTO, BCNN_VARIANT_VALU, BCNN_VARIANT_MFMA_I8, BCNN_VARIANT_MFMA_FP4 = 0, 1, 2, 3
BCNN_VARIANT_MFMA_FP4_T4, BCNN_VARIANT_MFMA_FP4_T7 = 4, 5
BCNN_VARIANT_MFMA_FP4_P6, BCNN_VARIANT_MFMA_FP4_P7, BCNN_VARIANT_MFMA_FP4_P5, BCNN_VARIANT_MFMA_FP4_P68 = 6, 7, 8, 9
BCNN_PAD_WORDS, BCNN_PAD_ZERO = 0, 1

EXPORTS = (
    "bcnn_pack", "bcnn_conv2d_binary", "bcnn_conv2d_binary_sign_pack",
    "bcnn_conv2d_binary_variant", "bcnn_threshold_sign_pack", "bcnn_out_dim",
    "bcnn_status_string", "bcnn_diag_copy_u32", "bcnn_diag_valu_peak",
    "bcnn_pack_bias", "bcnn_conv2d_binary_branches", "bcnn_conv2d_binary_branches_sign_pack",
    "bcnn_conv2d_binary_module", "bcnn_pack_bias_replicated", "bcnn_diag_mfma_fp4_peak",
    "bcnn_conv2d_binary_branches_module", "bcnn_avgpool_bias_sign_pack",
    "bcnn_diag_store_u32", "bcnn_diag_read_u32",
)


class bcnn_conv_desc(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in
                ("n", "c_in", "h", "w", "c_out", "kh", "kw", "stride", "pad")]


class bcnn_module_epilogue(ctypes.Structure):
    _fields_ = [("bn_scale", ctypes.c_void_p), ("bn_bias", ctypes.c_void_p), ("identity", ctypes.c_void_p),
                ("prelu_slope", ctypes.c_void_p), ("next_bias", ctypes.c_void_p), ("real_dtype", ctypes.c_int32),
                ("identity_channels", ctypes.c_int32)]


class BcnnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, bcnn_status_string(status), status))


_lib = None


def lib():
    """The loaded library.  Raises if libbcnn.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libbcnn.so is missing (%s): build it with `python -m paper_2010_00704_amd.build` "
                "or __graft_entry__.build(); there is no fallback path" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        dp = ctypes.POINTER(bcnn_conv_desc)
        L.bcnn_pack.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp]
        L.bcnn_conv2d_binary.argtypes = [dp, vp, vp, vp, vp]
        L.bcnn_conv2d_binary_sign_pack.argtypes = [dp, vp, vp, vp, vp, vp]
        L.bcnn_conv2d_binary_variant.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int, vp]
        L.bcnn_threshold_sign_pack.argtypes = [vp, vp, i64, i64, vp, vp]
        L.bcnn_out_dim.argtypes = [i32, i32, i32, i32]
        L.bcnn_status_string.argtypes = [ctypes.c_int]
        L.bcnn_status_string.restype = ctypes.c_char_p
        L.bcnn_diag_copy_u32.argtypes = [vp, vp, i64, vp]
        L.bcnn_diag_store_u32.argtypes = [vp, i64, i32, vp]
        L.bcnn_diag_read_u32.argtypes = [vp, i64, vp, i32, vp]
        L.bcnn_diag_valu_peak.argtypes = [vp, i32, i32, vp]
        L.bcnn_diag_mfma_fp4_peak.argtypes = [vp, i32, i32, vp]
        L.bcnn_pack_bias.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, vp, vp]
        L.bcnn_pack_bias_replicated.argtypes = [vp, ctypes.c_int, i64, i64, i64, i32, vp, vp, vp]
        L.bcnn_conv2d_binary_branches.argtypes = [dp, i32, vp, i64, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_int, vp]
        L.bcnn_conv2d_binary_branches_sign_pack.argtypes = [dp, i32, vp, i64, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_int, vp]
        L.bcnn_conv2d_binary_module.argtypes = [dp, vp, vp, ctypes.POINTER(bcnn_module_epilogue), vp, vp,
                                                ctypes.c_int, vp]
        L.bcnn_conv2d_binary_branches_module.argtypes = [
            dp, i32, vp, i64, vp, vp, ctypes.c_int, vp, vp, ctypes.POINTER(bcnn_module_epilogue), vp, vp,
            ctypes.c_int, vp]
        L.bcnn_avgpool_bias_sign_pack.argtypes = [vp, ctypes.c_int, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        for name in EXPORTS:
            if name != "bcnn_status_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(t):
    """Device address of a torch tensor (or a raw integer address / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _desc(d):
    if isinstance(d, bcnn_conv_desc):
        return d
    return bcnn_conv_desc(*[int(v) for v in d])


def bcnn_status_string(status):
    return lib().bcnn_status_string(int(status)).decode()


def bcnn_out_dim(size, k, stride, pad):
    return int(lib().bcnn_out_dim(size, k, stride, pad))


def bcnn_pack(src, dtype, outer, channels, inner, dst, stream=None):
    return lib().bcnn_pack(_ptr(src), dtype, outer, channels, inner, _ptr(dst), _stream(stream))


def bcnn_pack_bias(src, dtype, outer, channels, inner, bias, dst, stream=None):
    return lib().bcnn_pack_bias(_ptr(src), dtype, outer, channels, inner, _ptr(bias), _ptr(dst),
                                _stream(stream))


def bcnn_conv2d_binary_branches(desc, branches, x_packed, x_branch_stride, w_packed, pad_words, pad_mode,
                                scale, bias, z, variant=0, stream=None):
    return lib().bcnn_conv2d_binary_branches(ctypes.byref(_desc(desc)), int(branches), _ptr(x_packed),
                                             int(x_branch_stride), _ptr(w_packed),
                                             _ptr(pad_words), int(pad_mode), _ptr(scale), _ptr(bias),
                                             _ptr(z), int(variant), _stream(stream))


def bcnn_conv2d_binary_branches_sign_pack(desc, branches, x_packed, x_branch_stride, w_packed, pad_words,
                                          pad_mode, scale, bias, z_packed, variant=0, stream=None):
    return lib().bcnn_conv2d_binary_branches_sign_pack(
        ctypes.byref(_desc(desc)), int(branches), _ptr(x_packed), int(x_branch_stride),
        _ptr(w_packed), _ptr(pad_words), int(pad_mode), _ptr(scale), _ptr(bias), _ptr(z_packed),
        int(variant), _stream(stream))


def bcnn_pack_bias_replicated(src, dtype, outer, src_channels, inner, replication, bias, dst, stream=None):
    return lib().bcnn_pack_bias_replicated(_ptr(src), dtype, outer, src_channels, inner, int(replication),
                                           _ptr(bias), _ptr(dst), _stream(stream))


def bcnn_avgpool_bias_sign_pack(src, real_dtype, n, h, w, channels, s, bias, pooled, x_packed, stream=None):
    return lib().bcnn_avgpool_bias_sign_pack(_ptr(src), int(real_dtype), n, h, w, channels, s, _ptr(bias),
                                             _ptr(pooled), _ptr(x_packed), _stream(stream))


def bcnn_conv2d_binary_module(desc, x_packed, w_packed, bn_scale, bn_bias, identity, prelu_slope, next_bias,
                              real_dtype, r, x_next_packed, variant=0, stream=None, identity_channels=0):
    ep = bcnn_module_epilogue(_ptr(bn_scale), _ptr(bn_bias), _ptr(identity), _ptr(prelu_slope),
                              _ptr(next_bias), int(real_dtype), int(identity_channels))
    return lib().bcnn_conv2d_binary_module(ctypes.byref(_desc(desc)), _ptr(x_packed), _ptr(w_packed),
                                           ctypes.byref(ep), _ptr(r), _ptr(x_next_packed), int(variant),
                                           _stream(stream))


def bcnn_conv2d_binary_branches_module(desc, branches, x_packed, x_branch_stride, w_packed, pad_words, pad_mode,
                                       scale, bias, identity, prelu_slope, next_bias, real_dtype, r,
                                       x_next_packed, variant=0, stream=None, identity_channels=0):
    ep = bcnn_module_epilogue(None, None, _ptr(identity), _ptr(prelu_slope), _ptr(next_bias), int(real_dtype),
                              int(identity_channels))
    return lib().bcnn_conv2d_binary_branches_module(
        ctypes.byref(_desc(desc)), int(branches), _ptr(x_packed), int(x_branch_stride), _ptr(w_packed),
        _ptr(pad_words), int(pad_mode), _ptr(scale), _ptr(bias), ctypes.byref(ep), _ptr(r),
        _ptr(x_next_packed), int(variant), _stream(stream))


def bcnn_conv2d_binary(desc, x_packed, w_packed, y, stream=None):
    return lib().bcnn_conv2d_binary(ctypes.byref(_desc(desc)), _ptr(x_packed), _ptr(w_packed),
                                    _ptr(y), _stream(stream))


def bcnn_conv2d_binary_sign_pack(desc, x_packed, w_packed, thr, y_packed, stream=None):
    return lib().bcnn_conv2d_binary_sign_pack(ctypes.byref(_desc(desc)), _ptr(x_packed),
                                              _ptr(w_packed), _ptr(thr), _ptr(y_packed),
                                              _stream(stream))


def bcnn_conv2d_binary_variant(desc, x_packed, w_packed, thr, out, variant, stream=None):
    return lib().bcnn_conv2d_binary_variant(ctypes.byref(_desc(desc)), _ptr(x_packed),
                                            _ptr(w_packed), _ptr(thr), _ptr(out), int(variant),
                                            _stream(stream))


def bcnn_threshold_sign_pack(y, thr, rows, c_out, y_packed, stream=None):
    return lib().bcnn_threshold_sign_pack(_ptr(y), _ptr(thr), rows, c_out, _ptr(y_packed),
                                          _stream(stream))


def bcnn_diag_copy_u32(src, dst, words, stream=None):
    return lib().bcnn_diag_copy_u32(_ptr(src), _ptr(dst), words, _stream(stream))


def bcnn_diag_store_u32(dst, words, blocks=0, stream=None):
    return lib().bcnn_diag_store_u32(_ptr(dst), words, blocks, _stream(stream))


def bcnn_diag_read_u32(src, words, sink, blocks=0, stream=None):
    return lib().bcnn_diag_read_u32(_ptr(src), words, _ptr(sink), blocks, _stream(stream))


def bcnn_diag_valu_peak(sink, blocks, iters, stream=None):
    return lib().bcnn_diag_valu_peak(_ptr(sink), blocks, iters, _stream(stream))


def bcnn_diag_mfma_fp4_peak(sink, blocks, iters, stream=None):
    return lib().bcnn_diag_mfma_fp4_peak(_ptr(sink), blocks, iters, _stream(stream))


def check(status, where="bcnn"):
    if status != BCNN_OK:
        raise BcnnError(status, where)


# ---- conveniences that only allocate outputs with torch and call the above ----

_DTYPES = {torch.float32: BCNN_F32, torch.float16: BCNN_F16, torch.int8: BCNN_I8, torch.bfloat16: BCNN_BF16}


def pack_nchw(x, stream=None):
    """Device tensor [outer, C, *spatial] (f32/f16/i8) -> packed int32 tensor
    [outer, prod(spatial), ceil(C/32)] holding the uint32 words."""
    outer, c = x.shape[0], x.shape[1]
    inner = 1
    for d in x.shape[2:]:
        inner *= d
    out = torch.empty((outer, inner, (c + 31) // 32), dtype=torch.int32, device=x.device)
    check(bcnn_pack(x, _DTYPES[x.dtype], outer, c, inner, out, stream), "bcnn_pack")
    return out


def conv_desc(n, c_in, h, w, c_out, k, stride, pad):
    return bcnn_conv_desc(n, c_in, h, w, c_out, k, k, stride, pad)


def out_shape(desc):
    return (bcnn_out_dim(desc.h, desc.kh, desc.stride, desc.pad),
            bcnn_out_dim(desc.w, desc.kw, desc.stride, desc.pad))


def conv2d_binary(desc, x_packed, w_packed, variant=BCNN_VARIANT_AUTO, stream=None):
    """int32 sums [n, ho, wo, c_out]."""
    ho, wo = out_shape(desc)
    y = torch.empty((desc.n, ho, wo, desc.c_out), dtype=torch.int32, device=x_packed.device)
    check(bcnn_conv2d_binary_variant(desc, x_packed, w_packed, None, y, variant, stream),
          "bcnn_conv2d_binary")
    return y


def conv2d_binary_sign_pack(desc, x_packed, w_packed, thr, variant=BCNN_VARIANT_AUTO, stream=None):
    """packed bits [n, ho*wo, ceil(c_out/32)] (int32 storage of the uint32 words)."""
    ho, wo = out_shape(desc)
    yp = torch.empty((desc.n, ho * wo, (desc.c_out + 31) // 32), dtype=torch.int32,
                     device=x_packed.device)
    check(bcnn_conv2d_binary_variant(desc, x_packed, w_packed, thr, yp, variant, stream),
          "bcnn_conv2d_binary_sign_pack")
    return yp
