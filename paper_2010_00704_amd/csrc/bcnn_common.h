// Internal declarations shared by the HIP translation units of libbcnn.
// Nothing here is visible through the C ABI (include/bcnn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bcnn {

// Shape of one convolution call as the kernels see it.
struct ConvShape {
    int32_t n, h, w;        // input images and their extent
    int32_t cw;             // packed input words per pixel = ceil(c_in/32)
    int32_t c_out;
    int32_t cwo;            // packed output words per pixel = ceil(c_out/32)
    int32_t ks;             // filter extent, 1 or 3
    int32_t stride, pad;
    int32_t ho, wo;         // output extent
    int32_t m;              // n*ho*wo output pixels (rows of the GEMM view)
    int32_t k;              // c_in*ks*ks, the K of "dot = K - 2*popcount"
};

// Real-valued epilogue of a convolution module: batch-norm scale and bias,
// identity addition, PReLU, then the next module's bias and sign.
struct ModuleEp {
    const float* scale;      // [c_out]
    const float* bias;       // [c_out]
    const void* identity;    // [m][id_channels] float or half, or nullptr; channel o reads o mod id_channels
    int32_t id_channels;     // c_out unless the identity stream is replicated by bookkeeping
    const float* slope;      // [c_out] or nullptr (no activation)
    const float* next_bias;  // [c_out] or nullptr (0)
    void* r;                 // [m][c_out] float or half, or nullptr
    uint32_t* x_next;        // [m][cwo] packed bits of sign(r + next_bias), or nullptr
    int32_t half;            // type of identity and r: REAL_F32, REAL_F16 or REAL_BF16
};

// Storage type of a module's real stream (the paper fixes none; Section 4.2.1, first paragraph).
enum { REAL_F32 = 0, REAL_F16 = 1, REAL_BF16 = 2 };
template <int REAL> struct real_type { using type = float; };
template <> struct real_type<REAL_F16> { using type = _Float16; };
template <> struct real_type<REAL_BF16> { using type = __bf16; };

// One element of that epilogue: the order of operations is part of the
// interface (one rounding per step: fma, add, multiply; then storage
// rounding, to nearest even, when the stream is a 16-bit type).  Returns the value as stored.
template <int REAL>
__device__ __forceinline__ float module_tail(float t, bool has_id, float idv, bool has_slope, float a)
{
    if (has_id) t = t + idv;
    if (has_slope) t = (t >= 0.0f) ? t : a * t;
    if constexpr (REAL != REAL_F32) t = (float)(typename real_type<REAL>::type)t;
    return t;
}
template <int REAL>
__device__ __forceinline__ float module_value(float y, float g, float b, bool has_id, float idv,
                                              bool has_slope, float a)
{
    return module_tail<REAL>(__builtin_fmaf(g, y, b), has_id, idv, has_slope, a);
}

// Launchers, one per kernel family.  Each returns the hipError_t of its launch.
// bias: per-channel float added before the sign, or nullptr.  src_channels < channels: the source
// has src_channels channels and output channel c reads source channel c mod src_channels.
hipError_t launch_pack(const void* src, int dtype, const float* bias, int64_t outer, int64_t channels,
                       int64_t src_channels, int64_t inner, uint32_t* dst, hipStream_t stream);
hipError_t launch_threshold_sign_pack(const int32_t* y, const int32_t* thr, int64_t rows,
                                      int64_t c_out, uint32_t* y_packed, hipStream_t stream);
// ep != nullptr: module epilogue (thr and out are ignored)
hipError_t launch_conv_valu(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                            const int32_t* thr, void* out, const ModuleEp* ep, hipStream_t stream);
// fp4 matrix-core variant; `supported` says whether it covers the shape/alignment.
bool conv_mfma_fp4_supported(const ConvShape& s, const uint32_t* x, const uint32_t* w);
// whether the position-major tiling covers the shape (fused output only; see the launcher)
bool conv_mfma_fp4_pos_supported(const ConvShape& s);
// tile: pixel blocks per wave, 4 or 7 (7 exists for the fused kernel only), 0 = choose;
// 58, 67, 77: position-major tiles, 10 * (blocks per wave of interior tiles) + (of edge tiles), fused output only
hipError_t launch_conv_mfma_fp4(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                                const int32_t* thr, void* out, const ModuleEp* ep, int tile,
                                hipStream_t stream);
// int8 matrix-core variant (measurement arm, never chosen by AUTO)
bool conv_mfma_i8_supported(const ConvShape& s, const uint32_t* x, const uint32_t* w);
hipError_t launch_conv_mfma_i8(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                               const int32_t* thr, void* out, hipStream_t stream);
// Parallel 1x1 branches with per-branch real scales; F x F convolution as F*F
// shifted ones.
struct BranchArgs {
    int32_t branches;         // ks*ks (branch t reads the map shifted by tap t), or any count if ks == 1
    const uint32_t* x;        // packed activations, branch t at x + t * x_branch_stride
    int64_t x_branch_stride;  // in words; 0 = one tensor shared by all branches
    const uint32_t* w;        // packed weights [c_out][branches][cw]
    const uint32_t* pad_words;  // [branches][cw] operand of a tap outside the image, or nullptr (all -1)
    bool zero_pad;            // a tap outside the image contributes nothing
    const float* scale;       // [branches][c_out]
    const float* bias;        // [c_out] or nullptr
    void* out;                // float [m][c_out], or packed bits [m][cwo] when fused
    bool fused;
    // non-null: the branch sum continues into a module's tail (identity addition, PReLU, real stream
    // out, next bias + sign + pack); scale and bias of *tail are unused, `out` and `fused` too
    const ModuleEp* tail;
};
hipError_t launch_conv_branches(const ConvShape& s, const BranchArgs& a, hipStream_t stream);
// the same on the matrix cores; `supported` says whether it covers the call
bool conv_branches_mfma_supported(const ConvShape& s, const BranchArgs& a);
hipError_t launch_conv_branches_mfma(const ConvShape& s, const BranchArgs& a, hipStream_t stream);
// S x S / S average pooling of a channel-last real map [n][h][w][c] (of type REAL_* `real`), fused
// with bias + sign + pack of the pooled map; pooled or bits may be nullptr, bias too (zero)
hipError_t launch_avgpool_pack(const void* src, int real, int n, int h, int w, int c, int s, const float* bias,
                               void* pooled, uint32_t* bits, hipStream_t stream);

}  // namespace bcnn
