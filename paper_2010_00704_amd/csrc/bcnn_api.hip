// The C ABI of libbcnn (declared in include/bcnn.h): argument checks on the
// host, then one kernel launch on the caller's stream.  No allocation, no
// synchronisation, no state.
#include "bcnn.h"
#include "bcnn_common.h"

#include <limits.h>

namespace bcnn {
namespace {

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int out_dim(int in, int k, int stride, int pad)
{
    if (stride < 1 || k < 1 || pad < 0) return 0;
    const int span = in + 2 * pad - k;
    return span < 0 ? 0 : span / stride + 1;
}

// Fills `s` from the descriptor; returns BCNN_OK or the error to hand back.
int make_shape(const bcnn_conv_desc* d, ConvShape* s)
{
    if (!d) return BCNN_ERR_INVALID_ARG;
    if (d->n < 1 || d->c_in < 1 || d->h < 1 || d->w < 1 || d->c_out < 1) return BCNN_ERR_INVALID_ARG;
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0) return BCNN_ERR_INVALID_ARG;
    if (d->kh != d->kw || (d->kh != 1 && d->kh != 3)) return BCNN_ERR_UNSUPPORTED;
    if (d->stride > 2) return BCNN_ERR_UNSUPPORTED;
    if (d->pad > (d->kh - 1) / 2) return BCNN_ERR_UNSUPPORTED;
    const int ho = out_dim(d->h, d->kh, d->stride, d->pad);
    const int wo = out_dim(d->w, d->kw, d->stride, d->pad);
    if (ho < 1 || wo < 1) return BCNN_ERR_INVALID_ARG;
    const int64_t cw = ((int64_t)d->c_in + 31) / 32;
    const int64_t m = (int64_t)d->n * ho * wo;
    const int64_t k = (int64_t)d->c_in * d->kh * d->kw;
    if (m * d->c_out > INT_MAX || (int64_t)d->n * d->h * d->w * cw > INT_MAX || k > INT_MAX / 4 ||
        (int64_t)d->c_out * d->kh * d->kw * cw > INT_MAX)
        return BCNN_ERR_UNSUPPORTED;
    s->n = d->n; s->h = d->h; s->w = d->w; s->cw = (int32_t)cw;
    s->c_out = d->c_out; s->cwo = (d->c_out + 31) / 32;
    s->ks = d->kh; s->stride = d->stride; s->pad = d->pad;
    s->ho = ho; s->wo = wo; s->m = (int32_t)m; s->k = (int32_t)k;
    return BCNN_OK;
}

int conv_entry(const bcnn_conv_desc* desc, const uint32_t* x, const uint32_t* w, const int32_t* thr,
               bool fused, void* out, int variant, void* stream)
{
    ConvShape s;
    const int rc = make_shape(desc, &s);
    if (rc != BCNN_OK) return rc;
    if (!x || !w || !out || (fused && !thr)) return BCNN_ERR_INVALID_ARG;
    if (static_cast<const void*>(x) == out) return BCNN_ERR_INVALID_ARG;
    if (!aligned(x, 4) || !aligned(w, 4) || !aligned(out, 4) || (fused && !aligned(thr, 4)))
        return BCNN_ERR_ALIGNMENT;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (variant) {
        case BCNN_VARIANT_AUTO:
            // Measured over a grid of shapes (1x1 and 3x3, 128..1024 input and
            // 32..512 output channels, 49..200 000 pixels): wherever the matrix-core
            // kernel covers a shape it is faster than the vector-ALU kernel or within
            // half a microsecond of it, tiny problems included.
            if (conv_mfma_fp4_supported(s, x, w))
                e = launch_conv_mfma_fp4(s, x, w, fused ? thr : nullptr, out, nullptr, 0, st);
            else
                e = launch_conv_valu(s, x, w, fused ? thr : nullptr, out, nullptr, st);
            break;
        case BCNN_VARIANT_VALU:
            e = launch_conv_valu(s, x, w, fused ? thr : nullptr, out, nullptr, st);
            break;
        case BCNN_VARIANT_MFMA_FP4:
        case BCNN_VARIANT_MFMA_FP4_T4:
        case BCNN_VARIANT_MFMA_FP4_T7:
            if (!conv_mfma_fp4_supported(s, x, w)) return BCNN_ERR_UNSUPPORTED;
            if (variant == BCNN_VARIANT_MFMA_FP4_T7 && !fused) return BCNN_ERR_UNSUPPORTED;
            e = launch_conv_mfma_fp4(s, x, w, fused ? thr : nullptr, out, nullptr,
                                     variant == BCNN_VARIANT_MFMA_FP4_T7 ? 7 : variant == BCNN_VARIANT_MFMA_FP4_T4 ? 4 : 0, st);
            break;
        case BCNN_VARIANT_MFMA_FP4_P6:
        case BCNN_VARIANT_MFMA_FP4_P7:
        case BCNN_VARIANT_MFMA_FP4_P5:
        case BCNN_VARIANT_MFMA_FP4_P68:
            if (!fused || !conv_mfma_fp4_supported(s, x, w) || !conv_mfma_fp4_pos_supported(s)) return BCNN_ERR_UNSUPPORTED;
            e = launch_conv_mfma_fp4(s, x, w, thr, out, nullptr,
                                     variant == BCNN_VARIANT_MFMA_FP4_P6 ? 67 : variant == BCNN_VARIANT_MFMA_FP4_P7 ? 77 :
                                     variant == BCNN_VARIANT_MFMA_FP4_P68 ? 68 : 58, st);
            break;
        case BCNN_VARIANT_MFMA_I8:
            if (!conv_mfma_i8_supported(s, x, w)) return BCNN_ERR_UNSUPPORTED;
            e = launch_conv_mfma_i8(s, x, w, fused ? thr : nullptr, out, st);
            break;
        default:
            return BCNN_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

}  // namespace
}  // namespace bcnn

extern "C" {

int bcnn_out_dim(int32_t in, int32_t k, int32_t stride, int32_t pad)
{
    return bcnn::out_dim(in, k, stride, pad);
}

const char* bcnn_status_string(int status)
{
    switch (status) {
        case BCNN_OK: return "ok";
        case BCNN_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive extent or aliased buffers)";
        case BCNN_ERR_UNSUPPORTED: return "unsupported filter size, stride, padding, dtype or tensor size";
        case BCNN_ERR_ALIGNMENT: return "pointer not sufficiently aligned";
        case BCNN_ERR_DEVICE: return "HIP runtime error at kernel launch";
        default: return "unknown status";
    }
}

// bcnn_dtype of a real stream -> the kernels' REAL_* code
static int real_kind(int dtype)
{
    return dtype == BCNN_F16 ? bcnn::REAL_F16 : dtype == BCNN_BF16 ? bcnn::REAL_BF16 : bcnn::REAL_F32;
}

static int pack_entry(const void* src, int dtype, int64_t outer, int64_t channels, int64_t src_channels,
                      int64_t inner, const float* bias, uint32_t* dst, void* hip_stream)
{
    if (!src || !dst || outer < 1 || channels < 1 || inner < 1) return BCNN_ERR_INVALID_ARG;
    if (src_channels < 1 || src_channels > channels) return BCNN_ERR_INVALID_ARG;
    if (dtype != BCNN_F32 && dtype != BCNN_F16 && dtype != BCNN_I8 && dtype != BCNN_BF16) return BCNN_ERR_UNSUPPORTED;
    const int64_t cw = (channels + 31) / 32;
    if (outer > INT_MAX || inner > INT_MAX || outer * inner > INT_MAX / cw) return BCNN_ERR_UNSUPPORTED;
    if ((double)outer * (double)channels * (double)inner > 9.0e18) return BCNN_ERR_UNSUPPORTED;
    const uintptr_t esz = dtype == BCNN_F32 ? 4 : dtype == BCNN_I8 ? 1 : 2;
    if (!bcnn::aligned(src, esz) || !bcnn::aligned(dst, 4)) return BCNN_ERR_ALIGNMENT;
    if (src == static_cast<const void*>(dst)) return BCNN_ERR_INVALID_ARG;
    if (bias && !bcnn::aligned(bias, 4)) return BCNN_ERR_ALIGNMENT;
    const hipError_t e = bcnn::launch_pack(src, dtype, bias, outer, channels, src_channels, inner, dst,
                                           static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_pack(const void* src, bcnn_dtype dtype, int64_t outer, int64_t channels, int64_t inner,
              uint32_t* dst, void* hip_stream)
{
    return pack_entry(src, dtype, outer, channels, channels, inner, nullptr, dst, hip_stream);
}

int bcnn_pack_bias(const void* src, bcnn_dtype dtype, int64_t outer, int64_t channels, int64_t inner,
                   const float* bias, uint32_t* dst, void* hip_stream)
{
    if (!bias) return BCNN_ERR_INVALID_ARG;
    return pack_entry(src, dtype, outer, channels, channels, inner, bias, dst, hip_stream);
}

int bcnn_pack_bias_replicated(const void* src, bcnn_dtype dtype, int64_t outer, int64_t src_channels,
                              int64_t inner, int32_t replication, const float* bias, uint32_t* dst,
                              void* hip_stream)
{
    if (!bias || replication < 1 || src_channels < 1) return BCNN_ERR_INVALID_ARG;
    if (src_channels > INT_MAX / replication) return BCNN_ERR_UNSUPPORTED;
    return pack_entry(src, dtype, outer, src_channels * replication, src_channels, inner, bias, dst,
                      hip_stream);
}

int bcnn_avgpool_bias_sign_pack(const void* src, bcnn_dtype real_dtype, int32_t n, int32_t h, int32_t w,
                                int32_t channels, int32_t s, const float* bias, void* pooled,
                                uint32_t* x_packed, void* hip_stream)
{
    if (!src || (!pooled && !x_packed)) return BCNN_ERR_INVALID_ARG;
    if (n < 1 || h < 1 || w < 1 || channels < 1 || s < 1) return BCNN_ERR_INVALID_ARG;
    if (real_dtype != BCNN_F32 && real_dtype != BCNN_F16 && real_dtype != BCNN_BF16) return BCNN_ERR_UNSUPPORTED;
    if (s > 8) return BCNN_ERR_UNSUPPORTED;
    const int64_t ho = h / s, wo = w / s;
    if (ho < 1 || wo < 1) return BCNN_ERR_INVALID_ARG;
    const int64_t cw = (channels + 31) / 32;
    if ((double)n * (double)ho * (double)wo * 8.0 * (double)cw > (double)INT_MAX) return BCNN_ERR_UNSUPPORTED;
    const uintptr_t esz = real_dtype == BCNN_F32 ? 4 : 2;
    if (!bcnn::aligned(src, esz) || !bcnn::aligned(pooled, esz) || !bcnn::aligned(x_packed, 4) ||
        !bcnn::aligned(bias, 4))
        return BCNN_ERR_ALIGNMENT;
    if (src == pooled || src == static_cast<const void*>(x_packed)) return BCNN_ERR_INVALID_ARG;
    const hipError_t e = bcnn::launch_avgpool_pack(src, real_kind(real_dtype), n, h, w, channels, s, bias, pooled,
                                                   x_packed, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

static int branches_entry(const bcnn_conv_desc* desc, int32_t branches, const uint32_t* x,
                          int64_t x_branch_stride, const bcnn::ModuleEp* tail,
                          const uint32_t* w, const uint32_t* pad_words, int pad_mode,
                          const float* scale, const float* bias, void* out, bool fused, int variant,
                          void* hip_stream)
{
    bcnn::ConvShape s;
    const int rc = bcnn::make_shape(desc, &s);
    if (rc != BCNN_OK) return rc;
    if (!x || !w || !scale || (!out && !tail)) return BCNN_ERR_INVALID_ARG;
    if (tail && s.c_out < 32) return BCNN_ERR_UNSUPPORTED;
    if (pad_mode != BCNN_PAD_WORDS && pad_mode != BCNN_PAD_ZERO) return BCNN_ERR_INVALID_ARG;
    if (branches < 1 || (s.ks > 1 && branches != s.ks * s.ks)) return BCNN_ERR_INVALID_ARG;
    if (branches > 1024 || (int64_t)s.c_out * branches * s.cw > INT_MAX) return BCNN_ERR_UNSUPPORTED;
    const int64_t tensor_words = (int64_t)s.n * s.h * s.w * s.cw;
    if (x_branch_stride != 0 && x_branch_stride < tensor_words) return BCNN_ERR_INVALID_ARG;
    if (x_branch_stride * branches > INT_MAX) return BCNN_ERR_UNSUPPORTED;
    if (out && static_cast<const void*>(x) == out) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(x, 4) || !bcnn::aligned(w, 4) || !bcnn::aligned(scale, 4) || !bcnn::aligned(out, 4) ||
        (pad_words && !bcnn::aligned(pad_words, 4)) || (bias && !bcnn::aligned(bias, 4)))
        return BCNN_ERR_ALIGNMENT;
    bcnn::BranchArgs a;
    a.branches = branches;
    a.x = x; a.x_branch_stride = x_branch_stride; a.w = w;
    a.pad_words = pad_mode == BCNN_PAD_WORDS ? pad_words : nullptr;
    a.zero_pad = pad_mode == BCNN_PAD_ZERO;
    a.scale = scale; a.bias = bias; a.out = out; a.fused = fused; a.tail = tail;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const bool mfma_ok = bcnn::conv_branches_mfma_supported(s, a);
    hipError_t e;
    switch (variant) {
        case BCNN_VARIANT_AUTO:
            // measured: the matrix-core kernel wins at every size it covers
            if (mfma_ok) e = bcnn::launch_conv_branches_mfma(s, a, st);
            else e = bcnn::launch_conv_branches(s, a, st);
            break;
        case BCNN_VARIANT_VALU:
            e = bcnn::launch_conv_branches(s, a, st);
            break;
        case BCNN_VARIANT_MFMA_FP4:
            if (!mfma_ok) return BCNN_ERR_UNSUPPORTED;
            e = bcnn::launch_conv_branches_mfma(s, a, st);
            break;
        default:
            return BCNN_ERR_UNSUPPORTED;
    }
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_conv2d_binary_branches(const bcnn_conv_desc* desc, int32_t branches, const uint32_t* x_packed,
                                int64_t x_branch_stride, const uint32_t* w_packed,
                                const uint32_t* pad_words, int pad_mode, const float* scale,
                                const float* bias, float* z, int variant, void* hip_stream)
{
    return branches_entry(desc, branches, x_packed, x_branch_stride, nullptr, w_packed, pad_words, pad_mode,
                          scale, bias, z, false, variant, hip_stream);
}

int bcnn_conv2d_binary_branches_sign_pack(const bcnn_conv_desc* desc, int32_t branches,
                                          const uint32_t* x_packed, int64_t x_branch_stride, const uint32_t* w_packed,
                                          const uint32_t* pad_words, int pad_mode, const float* scale,
                                          const float* bias, uint32_t* z_packed, int variant,
                                          void* hip_stream)
{
    return branches_entry(desc, branches, x_packed, x_branch_stride, nullptr, w_packed, pad_words, pad_mode,
                          scale, bias, z_packed, true, variant, hip_stream);
}

// Fills the kernels' view of a module epilogue from the public struct; `with_bn` says whether the
// batch-norm scale and bias are part of this call.  Returns BCNN_OK or the error.
static int make_module_ep(const bcnn_module_epilogue* ep, bool with_bn, const bcnn::ConvShape& s,
                          const void* x_packed, void* r, uint32_t* x_next_packed, bcnn::ModuleEp* m)
{
    if (!ep || (with_bn && (!ep->bn_scale || !ep->bn_bias))) return BCNN_ERR_INVALID_ARG;
    if (!with_bn && (ep->bn_scale || ep->bn_bias)) return BCNN_ERR_INVALID_ARG;
    if (!r && !x_next_packed) return BCNN_ERR_INVALID_ARG;
    if (ep->real_dtype != BCNN_F32 && ep->real_dtype != BCNN_F16 && ep->real_dtype != BCNN_BF16)
        return BCNN_ERR_UNSUPPORTED;
    if (!with_bn && ep->real_dtype == BCNN_BF16) return BCNN_ERR_UNSUPPORTED;   // branch sums end in float or half
    const int id_channels = ep->identity_channels ? ep->identity_channels : s.c_out;
    if (id_channels < 1 || id_channels > s.c_out) return BCNN_ERR_INVALID_ARG;
    if (id_channels != s.c_out && ep->identity && ep->identity == r) return BCNN_ERR_INVALID_ARG;
    const uintptr_t esz = ep->real_dtype == BCNN_F32 ? 4 : 2;
    if (x_packed == static_cast<const void*>(x_next_packed) || x_packed == r) return BCNN_ERR_INVALID_ARG;
    if ((ep->bn_scale && !bcnn::aligned(ep->bn_scale, 4)) || (ep->bn_bias && !bcnn::aligned(ep->bn_bias, 4)) ||
        (ep->prelu_slope && !bcnn::aligned(ep->prelu_slope, 4)) ||
        (ep->next_bias && !bcnn::aligned(ep->next_bias, 4)) || (ep->identity && !bcnn::aligned(ep->identity, esz)) ||
        (r && !bcnn::aligned(r, esz)) || (x_next_packed && !bcnn::aligned(x_next_packed, 4)))
        return BCNN_ERR_ALIGNMENT;
    m->scale = ep->bn_scale; m->bias = ep->bn_bias; m->identity = ep->identity; m->slope = ep->prelu_slope;
    m->id_channels = id_channels;
    m->next_bias = ep->next_bias; m->r = r; m->x_next = x_next_packed; m->half = real_kind(ep->real_dtype);
    return BCNN_OK;
}

int bcnn_conv2d_binary_branches_module(const bcnn_conv_desc* desc, int32_t branches,
                                       const uint32_t* x_packed, int64_t x_branch_stride,
                                       const uint32_t* w_packed, const uint32_t* pad_words, int pad_mode,
                                       const float* scale, const float* bias,
                                       const bcnn_module_epilogue* ep, void* r, uint32_t* x_next_packed,
                                       int variant, void* hip_stream)
{
    bcnn::ConvShape s;
    const int rc = bcnn::make_shape(desc, &s);
    if (rc != BCNN_OK) return rc;
    bcnn::ModuleEp m;
    const int rc2 = make_module_ep(ep, false, s, x_packed, r, x_next_packed, &m);
    if (rc2 != BCNN_OK) return rc2;
    return branches_entry(desc, branches, x_packed, x_branch_stride, &m, w_packed, pad_words, pad_mode, scale,
                          bias, nullptr, false, variant, hip_stream);
}

int bcnn_conv2d_binary(const bcnn_conv_desc* desc, const uint32_t* x_packed,
                       const uint32_t* w_packed, int32_t* y, void* hip_stream)
{
    return bcnn::conv_entry(desc, x_packed, w_packed, nullptr, false, y, BCNN_VARIANT_AUTO, hip_stream);
}

int bcnn_conv2d_binary_sign_pack(const bcnn_conv_desc* desc, const uint32_t* x_packed,
                                 const uint32_t* w_packed, const int32_t* thr,
                                 uint32_t* y_packed, void* hip_stream)
{
    return bcnn::conv_entry(desc, x_packed, w_packed, thr, true, y_packed, BCNN_VARIANT_AUTO, hip_stream);
}

int bcnn_conv2d_binary_variant(const bcnn_conv_desc* desc, const uint32_t* x_packed,
                               const uint32_t* w_packed, const int32_t* thr, void* out,
                               int variant, void* hip_stream)
{
    return bcnn::conv_entry(desc, x_packed, w_packed, thr, thr != nullptr, out, variant, hip_stream);
}

int bcnn_conv2d_binary_module(const bcnn_conv_desc* desc, const uint32_t* x_packed,
                              const uint32_t* w_packed, const bcnn_module_epilogue* ep, void* r,
                              uint32_t* x_next_packed, int variant, void* hip_stream)
{
    bcnn::ConvShape s;
    const int rc = bcnn::make_shape(desc, &s);
    if (rc != BCNN_OK) return rc;
    if (!x_packed || !w_packed) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(x_packed, 4) || !bcnn::aligned(w_packed, 4)) return BCNN_ERR_ALIGNMENT;
    bcnn::ModuleEp m;
    const int rc2 = make_module_ep(ep, true, s, x_packed, r, x_next_packed, &m);
    if (rc2 != BCNN_OK) return rc2;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    const bool mfma_ok = bcnn::conv_mfma_fp4_supported(s, x_packed, w_packed);
    const int kwords = s.ks * s.ks * s.cw;      // packed words per output element
    switch (variant) {
        case BCNN_VARIANT_AUTO:
            // The module epilogue makes the matrix-core kernel's fixed cost about 10 us
            // against 7 us on the vector ALUs, whose time grows with the words per output
            // (taps x C_in / 32): measured on 1x1 and 3x3 modules, the matrix cores win at
            // every size from 16 words on, and below that from about 3e7 output elements x
            // words on.
            if (mfma_ok && (kwords >= 16 || (double)s.m * s.c_out * kwords >= 3.0e7))
                e = bcnn::launch_conv_mfma_fp4(s, x_packed, w_packed, nullptr, nullptr, &m, 0, st);
            else
                e = bcnn::launch_conv_valu(s, x_packed, w_packed, nullptr, nullptr, &m, st);
            break;
        case BCNN_VARIANT_VALU:
            e = bcnn::launch_conv_valu(s, x_packed, w_packed, nullptr, nullptr, &m, st);
            break;
        case BCNN_VARIANT_MFMA_FP4:
        case BCNN_VARIANT_MFMA_FP4_T4:
            if (!mfma_ok) return BCNN_ERR_UNSUPPORTED;
            e = bcnn::launch_conv_mfma_fp4(s, x_packed, w_packed, nullptr, nullptr, &m, 4, st);
            break;
        default:
            return BCNN_ERR_UNSUPPORTED;
    }
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_threshold_sign_pack(const int32_t* y, const int32_t* thr, int64_t rows, int64_t c_out,
                             uint32_t* y_packed, void* hip_stream)
{
    if (!y || !thr || !y_packed || rows < 1 || c_out < 1) return BCNN_ERR_INVALID_ARG;
    if (c_out > INT_MAX || rows > INT_MAX || rows * ((c_out + 31) / 32) > INT_MAX)
        return BCNN_ERR_UNSUPPORTED;
    if (!bcnn::aligned(y, 4) || !bcnn::aligned(thr, 4) || !bcnn::aligned(y_packed, 4))
        return BCNN_ERR_ALIGNMENT;
    if (static_cast<const void*>(y) == static_cast<const void*>(y_packed)) return BCNN_ERR_INVALID_ARG;
    const hipError_t e = bcnn::launch_threshold_sign_pack(y, thr, rows, c_out, y_packed,
                                                          static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

}  // extern "C"
