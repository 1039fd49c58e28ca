// S x S / S average pooling of the channel-last real stream, fused with the
// bias + sign + pack of the binary 1x1 convolution module behind it (BCNN
// paper, Section 4.2.3: identity path of a down-sampling block; Section 4.2.1,
// first paragraph: bias, then sign, in front of the binary convolution).
//
// One pass reads the S*S source vectors of an output element once and writes
// both consumers of the pooled map: the real map itself (the identity input of
// the module) and its packed sign bits (the module's binary operand).  HBM
// bound: S*S*esz bytes read, esz + 1/8 bytes written per output element.
//
// The arithmetic is fixed so that the bits are reproducible: the window's
// values are added in raster order in float32, one rounding per addition, the
// sum is divided by float(S*S), the quotient is stored (rounded to nearest
// even if the stream is half precision), and bit = (stored + bias >= 0) with
// the sum rounded to float32.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "bcnn_common.h"

namespace bcnn {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

struct PoolShape {
    int n, h, w, c, s, ho, wo;
    int cw;          // packed words per output pixel
    int units;       // vector kernel: output pixels * 8 * cw lanes of four channels (the caller keeps it below 2^31)
    int upp_shift;   // log2(8 * cw) when that is a power of two, else -1
};

__device__ __forceinline__ f4 load4(const float* p) { return *reinterpret_cast<const f4*>(p); }
__device__ __forceinline__ f4 load4(const __half* p)
{
    const uint2 raw = *reinterpret_cast<const uint2*>(p);
    const __half2 lo = *reinterpret_cast<const __half2*>(&raw.x);
    const __half2 hi = *reinterpret_cast<const __half2*>(&raw.y);
    return f4{__low2float(lo), __high2float(lo), __low2float(hi), __high2float(hi)};
}
__device__ __forceinline__ f4 load4(const __bf16* p)
{
    typedef __bf16 b4 __attribute__((ext_vector_type(4)));
    const b4 v = *reinterpret_cast<const b4*>(p);
    return f4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
}
// Stores the four values in the stream's type and returns them as stored.
__device__ __forceinline__ f4 round_and_store4(float* p, f4 v, bool store)
{
    if (store) *reinterpret_cast<f4*>(p) = v;
    return v;
}
__device__ __forceinline__ f4 round_and_store4(__half* p, f4 v, bool store)
{
    const __half2 lo = __halves2half2(__float2half_rn(v[0]), __float2half_rn(v[1]));
    const __half2 hi = __halves2half2(__float2half_rn(v[2]), __float2half_rn(v[3]));
    if (store) {
        uint2 raw;
        raw.x = *reinterpret_cast<const uint32_t*>(&lo);
        raw.y = *reinterpret_cast<const uint32_t*>(&hi);
        *reinterpret_cast<uint2*>(p) = raw;
    }
    return f4{__low2float(lo), __high2float(lo), __low2float(hi), __high2float(hi)};
}
__device__ __forceinline__ f4 round_and_store4(__bf16* p, f4 v, bool store)
{
    typedef __bf16 b4 __attribute__((ext_vector_type(4)));
    const b4 r = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};     // to nearest even
    if (store) *reinterpret_cast<b4*>(p) = r;
    return f4{(float)r[0], (float)r[1], (float)r[2], (float)r[3]};
}
__device__ __forceinline__ float as_float(float v) { return v; }
__device__ __forceinline__ float as_float(__bf16 v) { return (float)v; }
__device__ __forceinline__ float round_and_store1(__bf16* p, float v, bool store)
{
    const __bf16 r = (__bf16)v;
    if (store) *p = r;
    return (float)r;
}
__device__ __forceinline__ float as_float(__half v) { return __half2float(v); }
__device__ __forceinline__ float round_and_store1(float* p, float v, bool store)
{
    if (store) *p = v;
    return v;
}
__device__ __forceinline__ float round_and_store1(__half* p, float v, bool store)
{
    const __half hv = __float2half_rn(v);
    if (store) *p = hv;
    return __half2float(hv);
}

// Channels a multiple of 4, 16-byte (float) / 8-byte (half) aligned rows: a
// lane owns four consecutive channels of one output pixel, eight neighbouring
// lanes own the 32 channels of a packed word and OR their nibbles with three
// DPP exchanges.  Lanes past the last channel of a ragged last word idle.
// SF: window size known at compile time (all S*S loads in flight), 0 = p.s.
template <typename T, int SF>
__global__ __launch_bounds__(256) void avgpool_pack4_kernel(const T* __restrict__ src,
                                                            const float* __restrict__ bias, PoolShape p,
                                                            T* __restrict__ pooled, uint32_t* __restrict__ bits)
{
    // units per lane and round: small windows have few loads each, so a lane takes several units
    // (256 apart, which keeps the eight lanes of a word together) and issues all their loads first
    constexpr int U = SF == 1 ? 4 : SF == 2 ? 2 : 1;
    constexpr int NV = SF ? SF * SF : 1;
    const int s = SF ? SF : p.s;
    const float count = (float)(s * s);
    const int upp = 8 * p.cw;                       // lanes per output pixel
    const int lane8 = threadIdx.x & 7;
    const int64_t stride = (int64_t)gridDim.x * (256 * U);
    for (int64_t u0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x; u0 < p.units; u0 += stride) {
        f4 v[U][NV];
        int pixel[U], q[U];
        bool in[U], live[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int64_t u64 = u0 + 256 * k;
            in[k] = u64 < p.units;                  // the same for the eight lanes of a word
            const uint32_t u = in[k] ? (uint32_t)u64 : 0u;
            // the divisions below are most of this kernel's instructions for small windows: the common
            // cases (a power-of-two word count, a map that is one row of pixels) go without
            if (p.upp_shift >= 0) {
                pixel[k] = (int)(u >> p.upp_shift);
                q[k] = (int)(u & (uint32_t)(upp - 1));
            } else {
                pixel[k] = (int)(u / (uint32_t)upp);
                q[k] = (int)(u - (uint32_t)pixel[k] * (uint32_t)upp);
            }
            const int c0 = 4 * q[k];
            live[k] = in[k] && c0 < p.c;
            int n = pixel[k], oh = 0, ow = 0;
            if (p.ho != 1 || p.wo != 1) {
                const uint32_t rowo = (uint32_t)pixel[k] / (uint32_t)p.wo;
                ow = (int)((uint32_t)pixel[k] - rowo * (uint32_t)p.wo);
                n = (int)(rowo / (uint32_t)p.ho);
                oh = (int)(rowo - (uint32_t)n * (uint32_t)p.ho);
            }
            const T* win = src + (((int64_t)n * p.h + (int64_t)oh * s) * p.w + (int64_t)ow * s) * p.c + (live[k] ? c0 : 0);
            if constexpr (SF != 0) {
#pragma unroll
                for (int a = 0; a < SF; ++a)
#pragma unroll
                    for (int b = 0; b < SF; ++b) v[k][a * SF + b] = load4(win + ((int64_t)a * p.w + b) * p.c);
            } else {
                f4 acc = load4(win);
                for (int a = 0; a < s; ++a)
                    for (int b = (a == 0 ? 1 : 0); b < s; ++b) acc = acc + load4(win + ((int64_t)a * p.w + b) * p.c);
                v[k][0] = acc;
            }
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            f4 acc = v[k][0];
#pragma unroll
            for (int i = 1; i < NV; ++i) acc = acc + v[k][i];
            const f4 mean = acc / count;
            const int c0 = live[k] ? 4 * q[k] : 0;
            const f4 kept = round_and_store4(pooled + (int64_t)pixel[k] * p.c + c0, mean, live[k] && pooled);
            if (bits) {
                f4 b4 = f4{0.0f, 0.0f, 0.0f, 0.0f};
                if (bias && live[k]) b4 = load4(bias + c0);
                const f4 t = kept + b4;
                uint32_t w = ((uint32_t)(t[0] >= 0.0f) | ((uint32_t)(t[1] >= 0.0f) << 1) |
                              ((uint32_t)(t[2] >= 0.0f) << 2) | ((uint32_t)(t[3] >= 0.0f) << 3))
                             << (4 * lane8);
                w = live[k] ? w : 0u;
                // OR over the 8 lanes of the word: neighbours, pairs, then the other quad
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x141, 0xF, 0xF, true);  // row_half_mirror
                if (lane8 == 0 && in[k]) bits[(int64_t)pixel[k] * p.cw + (q[k] >> 3)] = w;
            }
        }
    }
}

// Any channel count and alignment: a wave takes 64 consecutive channels of one
// output pixel, lanes along channels; the wave-wide ballot is the word pair.
template <typename T>
__global__ __launch_bounds__(256) void avgpool_pack_kernel(const T* __restrict__ src,
                                                           const float* __restrict__ bias, PoolShape p,
                                                           T* __restrict__ pooled, uint32_t* __restrict__ bits)
{
    const int lane = threadIdx.x & 63;
    const int groups = (p.c + 63) / 64;
    const int64_t waves = (int64_t)p.n * p.ho * p.wo * groups;   // below 2^31 as well
    const int64_t stride = (int64_t)gridDim.x * 4;
    const float count = (float)(p.s * p.s);
    for (int64_t wv = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); wv < waves; wv += stride) {
        const int pixel = (int)wv / groups;
        const int g = (int)wv - pixel * groups;
        const int c = 64 * g + lane;
        const bool live = c < p.c;
        const int rowo = pixel / p.wo;
        const int ow = pixel - rowo * p.wo;
        const int n = rowo / p.ho;
        const int oh = rowo - n * p.ho;
        const T* win = src + (((int64_t)n * p.h + (int64_t)oh * p.s) * p.w + (int64_t)ow * p.s) * p.c + (live ? c : 0);
        float acc = as_float(win[0]);
        for (int a = 0; a < p.s; ++a)
            for (int b = (a == 0 ? 1 : 0); b < p.s; ++b) acc = acc + as_float(win[((int64_t)a * p.w + b) * p.c]);
        const float mean = acc / count;
        const float kept = round_and_store1(pooled + (int64_t)pixel * p.c + (live ? c : 0), mean, live && pooled);
        if (bits) {
            const float t = kept + ((bias && live) ? bias[c] : 0.0f);
            const uint64_t mask = __ballot(live && t >= 0.0f);
            if (lane < 2 && 2 * g + lane < p.cw) bits[(int64_t)pixel * p.cw + 2 * g + lane] = (uint32_t)(mask >> (32 * lane));
        }
    }
}

template <typename T>
hipError_t launch_typed(const T* src, const float* bias, PoolShape p, T* pooled, uint32_t* bits, hipStream_t stream)
{
    const uintptr_t vec = 4 * sizeof(T);
    const bool vector_ok = p.c % 4 == 0 && (reinterpret_cast<uintptr_t>(src) % vec) == 0 &&
                           (reinterpret_cast<uintptr_t>(pooled) % vec) == 0 &&
                           (reinterpret_cast<uintptr_t>(bias) % 16) == 0;
    const int64_t m = (int64_t)p.n * p.ho * p.wo;
    if (vector_ok) {
        p.units = (int)(m * 8 * p.cw);
        const int upl = p.s == 1 ? 4 : p.s == 2 ? 2 : 1;          // units per lane and round, as in the kernel
        const int64_t blocks = ((int64_t)p.units + 256 * upl - 1) / (256 * upl);   // one round per block
        const dim3 grid((unsigned)blocks), block(256);
        switch (p.s) {
        case 1: hipLaunchKernelGGL((avgpool_pack4_kernel<T, 1>), grid, block, 0, stream, src, bias, p, pooled, bits); break;
        case 2: hipLaunchKernelGGL((avgpool_pack4_kernel<T, 2>), grid, block, 0, stream, src, bias, p, pooled, bits); break;
        case 3: hipLaunchKernelGGL((avgpool_pack4_kernel<T, 3>), grid, block, 0, stream, src, bias, p, pooled, bits); break;
        case 4: hipLaunchKernelGGL((avgpool_pack4_kernel<T, 4>), grid, block, 0, stream, src, bias, p, pooled, bits); break;
        default: hipLaunchKernelGGL((avgpool_pack4_kernel<T, 0>), grid, block, 0, stream, src, bias, p, pooled, bits); break;
        }
        return hipGetLastError();
    }
    const int64_t waves = m * ((p.c + 63) / 64);
    int64_t blocks = (waves + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL((avgpool_pack_kernel<T>), dim3((unsigned)blocks), dim3(256), 0, stream, src, bias, p, pooled, bits);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_avgpool_pack(const void* src, int real, int n, int h, int w, int c, int s, const float* bias,
                               void* pooled, uint32_t* bits, hipStream_t stream)
{
    PoolShape p;
    p.n = n; p.h = h; p.w = w; p.c = c; p.s = s;
    p.ho = h / s; p.wo = w / s;
    p.cw = (c + 31) / 32;
    p.units = 0;
    p.upp_shift = -1;
    for (int sh = 3; sh < 31; ++sh)
        if ((8 * p.cw) == (1 << sh)) p.upp_shift = sh;
    if (real == REAL_F16)
        return launch_typed(static_cast<const __half*>(src), bias, p, static_cast<__half*>(pooled), bits, stream);
    if (real == REAL_BF16)
        return launch_typed(static_cast<const __bf16*>(src), bias, p, static_cast<__bf16*>(pooled), bits, stream);
    return launch_typed(static_cast<const float*>(src), bias, p, static_cast<float*>(pooled), bits, stream);
}

}  // namespace bcnn
