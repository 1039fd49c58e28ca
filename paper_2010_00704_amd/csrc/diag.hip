// Measurement helpers of libbcnn (declared in include/bcnn_diag.h): issue-rate
// probes of the vector ALUs and the matrix cores, and streaming kernels of known
// size (copy, store only, read only) that give memory-traffic counters and the
// HBM-bound kernels their denominators.  Not part of the method.
#include "bcnn.h"
#include "bcnn_diag.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bcnn {
namespace {

// Issue-rate probe: 64 independent accumulators per lane, each fed by one
// v_xor_b32 (scalar operand x vector operand, as in the convolution) and one
// v_bcnt_u32_b32 per round; operands live in registers only.  8 vector words
// times 8 scalar words give the 64 distinct pairs; the scalar words change
// every round so no xor can be hoisted out of the loop.
__global__ __launch_bounds__(256) void diag_valu_peak_kernel(uint32_t* __restrict__ sink, int iters)
{
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc[64];
#pragma unroll
    for (int a = 0; a < 64; ++a) acc[a] = 0;
    uint32_t xv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) xv[j] = (gid + j) * 2654435761u + 12345u;
    uint32_t sv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sv[j] = __builtin_amdgcn_readfirstlane(0x9E3779B9u * (j + 1));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) sv[j] = sv[j] * 5u + 1u;
#pragma unroll
        for (int a = 0; a < 64; ++a)
            acc[a] += __builtin_popcount(xv[a & 7] ^ sv[a >> 3]);
    }
    uint32_t r = 0;
#pragma unroll
    for (int a = 0; a < 64; ++a) r ^= acc[a];
    sink[gid] = r;
}

// Matrix-core issue-rate probe: every wave keeps 8 independent accumulators of
// v_mfma_f32_32x32x64_f8f6f4 busy with fp4 operands that are random +-1 (the
// codes 0x2 / 0xA, as in the convolution), held in registers; no memory traffic.
typedef int diag_v8i __attribute__((ext_vector_type(8)));
typedef float diag_v16f __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void diag_mfma_fp4_peak_kernel(float* __restrict__ sink, int iters)
{
    uint32_t seed = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    diag_v8i a[2], b[4];
    for (int q = 0; q < 6; ++q)
        for (int j = 0; j < 8; ++j) {
            seed = seed * 1664525u + 1013904223u;
            const int v = j < 4 ? (int)((seed & 0x88888888u) | 0x22222222u) : 0;
            if (q < 2) a[q][j] = v; else b[q - 2][j] = v;
        }
    diag_v16f c[8];
    for (int n = 0; n < 8; ++n)
        for (int r = 0; r < 16; ++r) c[n][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 8; ++n)
            c[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[n & 1], b[n >> 1], c[n], 4, 4, 0, 0, 0, 0);
    }
    float s = 0.0f;
    for (int n = 0; n < 8; ++n)
        for (int r = 0; r < 16; ++r) s += c[n][r];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void diag_copy_kernel(const uint32_t* __restrict__ src,
                                                       uint32_t* __restrict__ dst, int64_t words)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride)
        dst[i] = src[i];
}

// Store only: every lane writes 16-byte pieces (non-temporal, like the convolution's int32 output),
// a block covers UNROLL * 4 KB of consecutive bytes per round.
typedef uint32_t diag_u4 __attribute__((ext_vector_type(4)));
template <int UNROLL>
__global__ __launch_bounds__(256) void diag_store_kernel(diag_u4* __restrict__ dst, int64_t units, uint32_t value)
{
    const diag_u4 v = {value, value + 1u, value + 2u, value + 3u};
    const int64_t stride = (int64_t)gridDim.x * 256 * UNROLL;
    for (int64_t base = (int64_t)blockIdx.x * 256 * UNROLL + threadIdx.x; base < units; base += stride) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (base + 256 * u < units) __builtin_nontemporal_store(v, &dst[base + 256 * u]);
    }
}

// Read only: 16-byte non-temporal loads, UNROLL in flight per lane; the words are xor-ed together
// and one word per lane is written so that the loads cannot be dropped.
template <int UNROLL>
__global__ __launch_bounds__(256) void diag_read_kernel(const diag_u4* __restrict__ src, int64_t units,
                                                       uint32_t* __restrict__ sink)
{
    diag_u4 acc = {0u, 0u, 0u, 0u};
    const int64_t stride = (int64_t)gridDim.x * 256 * UNROLL;
    for (int64_t base = (int64_t)blockIdx.x * 256 * UNROLL + threadIdx.x; base < units; base += stride) {
        diag_u4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            v[u] = base + 256 * u < units ? __builtin_nontemporal_load(&src[base + 256 * u]) : diag_u4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
    }
    sink[blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace
}  // namespace bcnn

extern "C" {

int bcnn_diag_copy_u32(const uint32_t* src, uint32_t* dst, int64_t words, void* hip_stream)
{
    if (!src || !dst || words < 1) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(src, 4) || !bcnn::aligned(dst, 4)) return BCNN_ERR_ALIGNMENT;
    int64_t blocks = (words + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(bcnn::diag_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), src, dst, words);
    return hipGetLastError() == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_diag_store_u32(uint32_t* dst, int64_t words, int32_t blocks, void* hip_stream)
{
    if (!dst || words < 4 || words % 4 != 0 || blocks < 0) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(dst, 16)) return BCNN_ERR_ALIGNMENT;
    constexpr int UNROLL = 4;
    const int64_t units = words / 4;
    int64_t grid = blocks > 0 ? blocks : (units + 256 * UNROLL - 1) / (256 * UNROLL);
    if (grid > 0x7FFFFFFF) return BCNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((bcnn::diag_store_kernel<UNROLL>), dim3((unsigned)grid), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), reinterpret_cast<bcnn::diag_u4*>(dst), units, 0x01020304u);
    return hipGetLastError() == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_diag_read_u32(const uint32_t* src, int64_t words, uint32_t* sink, int32_t blocks, void* hip_stream)
{
    if (!src || !sink || words < 4 || words % 4 != 0 || blocks < 0) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(src, 16) || !bcnn::aligned(sink, 4)) return BCNN_ERR_ALIGNMENT;
    constexpr int UNROLL = 8;
    const int64_t units = words / 4;
    int64_t grid = blocks > 0 ? blocks : (units + 256 * UNROLL - 1) / (256 * UNROLL);
    if (grid > 0x7FFFFFFF) return BCNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((bcnn::diag_read_kernel<UNROLL>), dim3((unsigned)grid), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), reinterpret_cast<const bcnn::diag_u4*>(src), units, sink);
    return hipGetLastError() == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_diag_valu_peak(uint32_t* sink, int32_t blocks, int32_t iters, void* hip_stream)
{
    if (!sink || blocks < 1 || iters < 1) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(sink, 4)) return BCNN_ERR_ALIGNMENT;
    hipLaunchKernelGGL(bcnn::diag_valu_peak_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), sink, iters);
    return hipGetLastError() == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

int bcnn_diag_mfma_fp4_peak(float* sink, int32_t blocks, int32_t iters, void* hip_stream)
{
    if (!sink || blocks < 1 || iters < 1) return BCNN_ERR_INVALID_ARG;
    if (!bcnn::aligned(sink, 4)) return BCNN_ERR_ALIGNMENT;
    hipLaunchKernelGGL(bcnn::diag_mfma_fp4_peak_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), sink, iters);
    return hipGetLastError() == hipSuccess ? BCNN_OK : BCNN_ERR_DEVICE;
}

}  // extern "C"
