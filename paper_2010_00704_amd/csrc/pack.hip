// Sign-binarise + channel-pack kernels and the stand-alone threshold epilogue
// (BCNN paper, Section 4.2.1: sign before every binary convolution; Section
// 2.4: storage scales with the number of bits).  Both are pure streaming
// kernels: 4 bytes (or 2, or 1) read and 1 bit written per element, so HBM
// bandwidth is the only bound and the design goal is wide, coalesced reads
// with many of them in flight.
#include "bcnn_common.h"

#include <type_traits>


namespace bcnn {
namespace {

__device__ __forceinline__ bool nonneg(float v) { return v >= 0.0f; }
__device__ __forceinline__ bool nonneg(_Float16 v) { return (float)v >= 0.0f; }
__device__ __forceinline__ bool nonneg(__bf16 v) { return (float)v >= 0.0f; }
__device__ __forceinline__ bool nonneg(int8_t v) { return v >= 0; }

// The bit of one element: sign of the value, or (BIAS) of value + bias[channel]
// with the sum rounded to float (Section 4.2.1: learnable bias, then sign).
template <bool BIAS, typename T>
__device__ __forceinline__ bool bit_of(T v, const float* __restrict__ bias, int64_t c)
{
    if constexpr (BIAS) return (float)v + bias[c] >= 0.0f;
    else return nonneg(v);
}

// Channel replication by bookkeeping (Section 4.2.2 of the paper: a building
// block that widens the network sees every real channel R times; no copy of the
// real map is made): output channel c reads source channel c mod src_channels,
// while the bias stays indexed by c.  REP == false: src_channels == channels.
template <bool REP>
__device__ __forceinline__ int64_t src_channel(int64_t c, int64_t src_channels)
{
    if constexpr (REP) return (int64_t)((uint32_t)c % (uint32_t)src_channels);   // both below 2^31
    else return c;
}

// ---- [outer][C][inner] with inner >= 64: lanes run along `inner` ------------
// One thread owns one inner position and builds `cwg` consecutive words of that
// pixel.  For a fixed channel the 256 threads of a block read 256 consecutive
// elements; the 32 channel reads of a word are independent and all in flight.
// The block's words are staged through LDS so that each pixel's words leave
// in one contiguous run.  The channel words are split over blocks (cwg per
// block) until the launch has enough blocks to fill the chip.
constexpr int PACK_THREADS = 256;
constexpr int PACK_CW_CHUNK = 8;  // most words per block: 256*8*4 B = 8 KB LDS

template <typename T, bool BIAS, bool REP>
__global__ __launch_bounds__(PACK_THREADS) void pack_columns_kernel(
    const T* __restrict__ src, const float* __restrict__ bias, int64_t channels, int64_t src_channels,
    int64_t inner, int64_t cw_total, int cwg, int groups, uint32_t* __restrict__ dst)
{
    __shared__ uint32_t stage[PACK_THREADS * PACK_CW_CHUNK];
    const int64_t a = blockIdx.y / groups;
    const int64_t j0 = (int64_t)(blockIdx.y % groups) * cwg;
    const int64_t i0 = (int64_t)blockIdx.x * PACK_THREADS;
    const int tid = threadIdx.x;
    const int64_t i = i0 + tid;
    const bool live = i < inner;
    const int64_t icl = live ? i : inner - 1;
    const T* col = src + a * src_channels * inner + icl;
    const int rows_here = (int)((inner - i0 < PACK_THREADS) ? (inner - i0) : PACK_THREADS);
    const int jn = (int)((cw_total - j0 < cwg) ? (cw_total - j0) : cwg);

    for (int j = 0; j < jn; ++j) {
        const int64_t c0 = (j0 + j) * 32;
        uint32_t word = 0;
        if (c0 + 32 <= channels) {
            T v[32];
#pragma unroll
            for (int b = 0; b < 32; ++b)
                v[b] = __builtin_nontemporal_load(col + src_channel<REP>(c0 + b, src_channels) * inner);
#pragma unroll
            for (int b = 0; b < 32; ++b) word |= (uint32_t)bit_of<BIAS>(v[b], bias, c0 + b) << b;
        } else {
            for (int b = 0; c0 + b < channels; ++b)
                word |= (uint32_t)bit_of<BIAS>(col[src_channel<REP>(c0 + b, src_channels) * inner], bias, c0 + b) << b;
        }
        stage[tid * jn + j] = word;
    }
    __syncthreads();
    // rows_here*jn words: word t of the stage belongs to pixel t/jn, word t%jn of the group
    const int total = rows_here * jn;
    for (int t = tid; t < total; t += PACK_THREADS) {
        const int r = t / jn, j = t - r * jn;
        dst[(a * inner + i0 + r) * cw_total + j0 + j] = stage[t];
    }
}

// ---- fp32, inner a multiple of 4: four pixels per thread, whole rows per block ----
// The pixels of all images are numbered through (pixel a*inner + i is unit (a*inner + i) / 4, lane
// position i % 4), so every lane of every wave has work whatever `inner` is.  A block owns 64
// units = 256 consecutive output pixels and builds ALL packed words of them: wave w takes the
// words w, w+4, ... (up to PACK4_WORDS per block; more channels go to further blocks along y), 32
// independent 16-byte non-temporal loads per word in two batches of 16.  The words meet in LDS and leave
// as one contiguous run of 256 * words * 4 bytes: whole cache lines, written once.
constexpr int PACK4_WORDS = 32;   // packed words per pixel and block: 256 * 32 * 4 B = 32 KB of LDS

template <bool BIAS, bool REP>
__global__ __launch_bounds__(PACK_THREADS) void pack_units4_kernel(
    const float* __restrict__ src, const float* __restrict__ bias, int64_t channels, int64_t src_channels,
    int64_t inner, int64_t units, int64_t cw_total, uint32_t* __restrict__ dst)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    extern __shared__ uint32_t stage[];               // [256 pixels][jn words]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t j0 = (int64_t)blockIdx.y * PACK4_WORDS;
    const int jn = (int)((cw_total - j0 < PACK4_WORDS) ? (cw_total - j0) : PACK4_WORDS);
    const int64_t u0 = (int64_t)blockIdx.x * 64;
    const int64_t u = u0 + lane < units ? u0 + lane : units - 1;       // clamped: duplicates, not stored
    const int64_t per_image = inner >> 2;
    const int64_t a = u / per_image;
    const float* col = src + a * src_channels * inner + 4 * (u - a * per_image);

    for (int j = wave; j < jn; j += 4) {
        const int64_t c0 = (j0 + j) * 32;
        uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
        if (c0 + 32 <= channels) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {      // two batches of 16 loads: 64 registers in flight
                f4 v[16];
#pragma unroll
                for (int b = 0; b < 16; ++b)
                    v[b] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(
                        col + src_channel<REP>(c0 + 16 * half + b, src_channels) * inner));
#pragma unroll
                for (int b = 0; b < 16; ++b) {
                    w0 |= (uint32_t)bit_of<BIAS>(v[b][0], bias, c0 + 16 * half + b) << (16 * half + b);
                    w1 |= (uint32_t)bit_of<BIAS>(v[b][1], bias, c0 + 16 * half + b) << (16 * half + b);
                    w2 |= (uint32_t)bit_of<BIAS>(v[b][2], bias, c0 + 16 * half + b) << (16 * half + b);
                    w3 |= (uint32_t)bit_of<BIAS>(v[b][3], bias, c0 + 16 * half + b) << (16 * half + b);
                }
            }
        } else {
            for (int b = 0; c0 + b < channels; ++b) {
                const f4 v = *reinterpret_cast<const f4*>(col + src_channel<REP>(c0 + b, src_channels) * inner);
                w0 |= (uint32_t)bit_of<BIAS>(v[0], bias, c0 + b) << b;
                w1 |= (uint32_t)bit_of<BIAS>(v[1], bias, c0 + b) << b;
                w2 |= (uint32_t)bit_of<BIAS>(v[2], bias, c0 + b) << b;
                w3 |= (uint32_t)bit_of<BIAS>(v[3], bias, c0 + b) << b;
            }
        }
        stage[(4 * lane + 0) * jn + j] = w0;
        stage[(4 * lane + 1) * jn + j] = w1;
        stage[(4 * lane + 2) * jn + j] = w2;
        stage[(4 * lane + 3) * jn + j] = w3;
    }
    __syncthreads();
    // pixel 4*u0 + r, word j0 + j; rows of a block that owns every word are contiguous in dst
    const int64_t live = units - u0 < 64 ? units - u0 : 64;
    const int total = (int)(4 * live) * jn;
    uint32_t* out = dst + 4 * u0 * cw_total + j0;
    if (jn == cw_total) {
        for (int t = threadIdx.x; t < total; t += PACK_THREADS) out[t] = stage[t];
    } else {
        for (int t = threadIdx.x; t < total; t += PACK_THREADS) {
            const int r = t / jn, j = t - r * jn;
            out[(int64_t)r * cw_total + j] = stage[t];
        }
    }
}

// ---- 1 < inner < 64 (7x7 feature maps, 3x3 filter taps): 2D thread tile ------
// IP = inner rounded up to a power of two; thread (i = t % IP, q = t / IP)
// reads element i of channel rows q, q+R, q+2R, ... (R = 256/IP rows per pass:
// consecutive rows are contiguous in memory, so a pass reads R*inner
// consecutive elements).  A thread ORs its rows' sign bits into partial words,
// the R partials of a pixel meet in LDS.  A block packs up to 8 words (256
// channels) of one `outer` index.
template <typename T, int IP, bool BIAS, bool REP>
__global__ __launch_bounds__(256) void pack_small_inner_kernel(
    const T* __restrict__ src, const float* __restrict__ bias, int64_t channels, int64_t src_channels,
    int inner, int64_t cw_total, int groups, uint32_t* __restrict__ dst)
{
    constexpr int R = 256 / IP;          // channel rows per pass
    constexpr int PASSES = 32 / R;       // passes per output word (R divides 32 as IP >= 8)
    constexpr int G = 8;                 // words per block
    __shared__ uint32_t part[G][R][IP];
    const int64_t a = blockIdx.x / groups;
    const int64_t j0 = (int64_t)(blockIdx.x % groups) * G;
    const int i = threadIdx.x % IP, q = threadIdx.x / IP;
    const bool live = i < inner;
    const T* base = src + a * src_channels * inner + (live ? i : 0);
    const int jn = (int)((cw_total - j0 < G) ? (cw_total - j0) : G);
    for (int j = 0; j < jn; ++j) {
        const int64_t c0 = (j0 + j) * 32;
        uint32_t word = 0;
        if (c0 + 32 <= channels) {
            T v[PASSES];
#pragma unroll
            for (int k = 0; k < PASSES; ++k)
                v[k] = __builtin_nontemporal_load(base + src_channel<REP>(c0 + q + R * k, src_channels) * inner);
#pragma unroll
            for (int k = 0; k < PASSES; ++k)
                word |= (uint32_t)bit_of<BIAS>(v[k], bias, c0 + q + R * k) << (q + R * k);
        } else {
            for (int k = 0; k < PASSES; ++k) {
                const int64_t c = c0 + q + R * k;
                if (c < channels)
                    word |= (uint32_t)bit_of<BIAS>(base[src_channel<REP>(c, src_channels) * inner], bias, c) << (q + R * k);
            }
        }
        part[j][q][i] = live ? word : 0u;
    }
    __syncthreads();
    // thread t -> (pixel t / jn, word t % jn): each pixel's words leave together
    for (int t = threadIdx.x; t < inner * jn; t += 256) {
        const int px = t / jn, j = t - px * jn;
        uint32_t word = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) word |= part[j][r][px];
        dst[(a * inner + px) * cw_total + j0 + j] = word;
    }
}

// ---- inner == 1 (channel-last rows): lanes run along the channels ----------
// One wave per (row, 64-channel group); the wave-wide ballot IS the two packed
// words.  Reads are perfectly coalesced.  ROWS rows are handled per wave so
// that several loads are in flight.
template <typename T, int ROWS, bool BIAS, bool REP>
__global__ __launch_bounds__(256) void pack_rows_kernel(
    const T* __restrict__ src, const float* __restrict__ bias, int64_t rows, int64_t channels,
    int64_t src_channels, int64_t cw_total, uint32_t* __restrict__ dst)
{
    const int lane = threadIdx.x & 63;
    const int64_t groups = (channels + 63) / 64;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t g = wave % groups;
    const int64_t r0 = (wave / groups) * ROWS;
    if (r0 >= rows) return;
    const int64_t c = g * 64 + lane;
    bool bit[ROWS];
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const int64_t r = r0 + k;
        bit[k] = (r < rows && c < channels)
                     ? bit_of<BIAS>(src[r * src_channels + src_channel<REP>(c, src_channels)], bias, c) : false;
    }
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const uint64_t mask = __ballot(bit[k]);
        const int64_t r = r0 + k;
        if (r < rows && lane < 2 && g * 2 + lane < cw_total)
            dst[r * cw_total + g * 2 + lane] = (uint32_t)(mask >> (32 * lane));
    }
}

// ---- anything else (small inner, e.g. 3x3 filter taps): one thread per word --
template <typename T, bool BIAS, bool REP>
__global__ __launch_bounds__(256) void pack_generic_kernel(
    const T* __restrict__ src, const float* __restrict__ bias, int64_t outer, int64_t channels,
    int64_t src_channels, int64_t inner, int64_t cw_total, uint32_t* __restrict__ dst)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= outer * inner * cw_total) return;
    const int64_t j = t % cw_total;
    const int64_t i = (t / cw_total) % inner;
    const int64_t a = t / (cw_total * inner);
    uint32_t word = 0;
    for (int b = 0; b < 32; ++b) {
        const int64_t c = j * 32 + b;
        if (c < channels)
            word |= (uint32_t)bit_of<BIAS>(src[(a * src_channels + src_channel<REP>(c, src_channels)) * inner + i],
                                           bias, c) << b;
    }
    dst[t] = word;
}

template <typename T, bool BIAS, bool REP>
hipError_t pack_dispatch(const T* src, const float* bias, int64_t outer, int64_t channels,
                         int64_t src_channels, int64_t inner, uint32_t* dst, hipStream_t stream)
{
    const int64_t cw = (channels + 31) / 32;
    if (inner == 1) {
        constexpr int ROWS = 8;
        const int64_t groups = (channels + 63) / 64;
        const int64_t waves = ((outer + ROWS - 1) / ROWS) * groups;
        const int64_t blocks = (waves + 3) / 4;
        hipLaunchKernelGGL((pack_rows_kernel<T, ROWS, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           src, bias, outer, channels, src_channels, cw, dst);
    } else if (std::is_same<T, float>::value && inner >= 64 && inner % 4 == 0 && outer * (inner / 4) >= 64 * 128 &&
               (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
        // (from 128 blocks on; smaller inputs spread better over the chip with one pixel per thread)
        const int64_t units = outer * (inner / 4);
        const int64_t bx = (units + 63) / 64;
        const int64_t by = (cw + PACK4_WORDS - 1) / PACK4_WORDS;
        if (bx > 0x7FFFFFFF || by > 65535) goto generic;
        const int words = (int)(cw < PACK4_WORDS ? cw : PACK4_WORDS);
        hipLaunchKernelGGL((pack_units4_kernel<BIAS, REP>), dim3((unsigned)bx, (unsigned)by), dim3(PACK_THREADS),
                           (size_t)256 * words * 4, stream, reinterpret_cast<const float*>(src), bias, channels,
                           src_channels, inner, units, cw, dst);
    } else if (inner >= 64) {
        const int64_t bx = (inner + PACK_THREADS - 1) / PACK_THREADS;
        // words per block: as many as possible (up to 8) while two blocks per CU remain
        int cwg = PACK_CW_CHUNK;
        while (cwg > 1 && bx * outer * ((cw + cwg - 1) / cwg) < 512) cwg >>= 1;
        const int64_t groups = (cw + cwg - 1) / cwg;
        if (outer * groups > 65535) goto generic;
        hipLaunchKernelGGL((pack_columns_kernel<T, BIAS, REP>), dim3((unsigned)bx, (unsigned)(outer * groups)),
                           dim3(PACK_THREADS), 0, stream, src, bias, channels, src_channels, inner, cw, cwg,
                           (int)groups, dst);
    } else if (inner >= 5) {
        const int64_t groups = (cw + 7) / 8;
        const int64_t blocks = outer * groups;
        if (blocks > 0x7FFFFFFF) goto generic;
        if (inner > 32)
            hipLaunchKernelGGL((pack_small_inner_kernel<T, 64, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                               src, bias, channels, src_channels, (int)inner, cw, (int)groups, dst);
        else if (inner > 16)
            hipLaunchKernelGGL((pack_small_inner_kernel<T, 32, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                               src, bias, channels, src_channels, (int)inner, cw, (int)groups, dst);
        else if (inner > 8)
            hipLaunchKernelGGL((pack_small_inner_kernel<T, 16, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                               src, bias, channels, src_channels, (int)inner, cw, (int)groups, dst);
        else
            hipLaunchKernelGGL((pack_small_inner_kernel<T, 8, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                               src, bias, channels, src_channels, (int)inner, cw, (int)groups, dst);
    } else {
    generic:
        const int64_t total = outer * inner * cw;
        const int64_t blocks = (total + 255) / 256;
        hipLaunchKernelGGL((pack_generic_kernel<T, BIAS, REP>), dim3((unsigned)blocks), dim3(256), 0, stream,
                           src, bias, outer, channels, src_channels, inner, cw, dst);
    }
    return hipGetLastError();
}

// ---- stand-alone epilogue: int32 sums [rows][c_out] -> packed bits ---------
template <int ROWS>
__global__ __launch_bounds__(256) void threshold_sign_pack_kernel(
    const int32_t* __restrict__ y, const int32_t* __restrict__ thr, int64_t rows, int64_t c_out,
    int64_t cwo, uint32_t* __restrict__ yp)
{
    const int lane = threadIdx.x & 63;
    const int64_t groups = (c_out + 63) / 64;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t g = wave % groups;
    const int64_t r0 = (wave / groups) * ROWS;
    if (r0 >= rows) return;
    const int64_t c = g * 64 + lane;
    const bool cl = c < c_out;
    const int32_t t = cl ? thr[c] : 0;
    int32_t v[ROWS];
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const int64_t r = r0 + k;
        v[k] = (r < rows && cl) ? __builtin_nontemporal_load(y + r * c_out + c) : 0;
    }
#pragma unroll
    for (int k = 0; k < ROWS; ++k) {
        const uint64_t mask = __ballot(cl && v[k] >= t);
        const int64_t r = r0 + k;
        if (r < rows && lane < 2 && g * 2 + lane < cwo)
            yp[r * cwo + g * 2 + lane] = (uint32_t)(mask >> (32 * lane));
    }
}

// The same for c_out a multiple of 32 and 16-byte aligned sums: the tensor is
// a flat stream of 16-byte units (4 channels of one row), a lane takes UNROLL
// units per round with non-temporal 16-byte loads, eight neighbouring lanes
// hold the 32 channels of one output word and combine their nibbles with three
// DPP exchanges.
template <int UNROLL>
__global__ __launch_bounds__(256) void threshold_sign_pack4_kernel(
    const int32_t* __restrict__ y, const int32_t* __restrict__ thr, int64_t units, int c_out,
    uint32_t* __restrict__ yp)
{
    typedef int i4 __attribute__((ext_vector_type(4)));
    const int lane8 = threadIdx.x & 7;
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    // channel of this lane's unit, kept up to date by adding the stride modulo c_out
    int c = (int)((u * 4) % c_out);
    const int cstep = (int)((stride * 4) % c_out);
    for (; u < units; u += stride * UNROLL) {
        i4 v[UNROLL], t[UNROLL];
        int cc = c;
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            const int64_t uk = u + stride * k;
            const bool ok = uk < units;
            v[k] = ok ? __builtin_nontemporal_load(reinterpret_cast<const i4*>(y) + uk) : i4{0, 0, 0, 0};
            t[k] = *reinterpret_cast<const i4*>(thr + cc);
            cc += cstep; cc -= cc >= c_out ? c_out : 0;
        }
        c = cc;
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            const int64_t uk = u + stride * k;
            uint32_t w = ((uint32_t)(v[k][0] >= t[k][0]) | ((uint32_t)(v[k][1] >= t[k][1]) << 1) |
                          ((uint32_t)(v[k][2] >= t[k][2]) << 2) | ((uint32_t)(v[k][3] >= t[k][3]) << 3))
                         << (4 * lane8);
            // OR over the 8 lanes of the word: neighbours, pairs, then the other quad
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x141, 0xF, 0xF, true);  // row_half_mirror
            if (lane8 == 0 && uk < units) yp[uk >> 3] = w;
        }
    }
}

}  // namespace

template <typename T>
hipError_t pack_typed(const void* src, const float* bias, int64_t outer, int64_t channels,
                      int64_t src_channels, int64_t inner, uint32_t* dst, hipStream_t stream)
{
    const T* p = static_cast<const T*>(src);
    if (src_channels != channels)   // replication always comes with a bias
        return pack_dispatch<T, true, true>(p, bias, outer, channels, src_channels, inner, dst, stream);
    if (bias) return pack_dispatch<T, true, false>(p, bias, outer, channels, channels, inner, dst, stream);
    return pack_dispatch<T, false, false>(p, nullptr, outer, channels, channels, inner, dst, stream);
}

hipError_t launch_pack(const void* src, int dtype, const float* bias, int64_t outer, int64_t channels,
                       int64_t src_channels, int64_t inner, uint32_t* dst, hipStream_t stream)
{
    // A channel-last source (inner = 1) with whole 16-byte (float) / 8-byte (half) groups of four
    // channels is the pooling kernel's case with a 1 x 1 window: a lane takes four channels of a row,
    // eight lanes make a packed word.  Twice to three times the rate of the lanes-along-channels kernel.
    if (inner == 1 && src_channels == channels && (dtype == 0 || dtype == 1) && channels % 4 == 0 &&
        outer * 8 * ((channels + 31) / 32) <= 0x7FFFFFFF &&
        (reinterpret_cast<uintptr_t>(src) % (dtype == 0 ? 16 : 8)) == 0 &&
        (reinterpret_cast<uintptr_t>(bias) % 16) == 0)
        return launch_avgpool_pack(src, dtype == 1 ? REAL_F16 : REAL_F32, (int)outer, 1, 1, (int)channels, 1, bias, nullptr,
                                   dst, stream);
    switch (dtype) {
        case 0: return pack_typed<float>(src, bias, outer, channels, src_channels, inner, dst, stream);
        case 1: return pack_typed<_Float16>(src, bias, outer, channels, src_channels, inner, dst, stream);
        case 2: return pack_typed<int8_t>(src, bias, outer, channels, src_channels, inner, dst, stream);
        case 3: return pack_typed<__bf16>(src, bias, outer, channels, src_channels, inner, dst, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_threshold_sign_pack(const int32_t* y, const int32_t* thr, int64_t rows,
                                      int64_t c_out, uint32_t* y_packed, hipStream_t stream)
{
    if (c_out % 32 == 0 && ((reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(thr)) & 15) == 0) {
        constexpr int UNROLL = 4;
        const int64_t units = rows * (c_out / 4);
        // one round per block: blocks that finish early make room for the rest, so the tail stays short
        // (the kernel's loop only matters beyond 2^31 - 1 blocks, which the row limit excludes)
        const int64_t blocks = (units + 256 * UNROLL - 1) / (256 * UNROLL);
        hipLaunchKernelGGL((threshold_sign_pack4_kernel<UNROLL>), dim3((unsigned)blocks), dim3(256), 0,
                           stream, y, thr, units, (int)c_out, y_packed);
        return hipGetLastError();
    }
    constexpr int ROWS = 8;
    const int64_t groups = (c_out + 63) / 64;
    const int64_t waves = ((rows + ROWS - 1) / ROWS) * groups;
    const int64_t blocks = (waves + 3) / 4;
    hipLaunchKernelGGL((threshold_sign_pack_kernel<ROWS>), dim3((unsigned)blocks), dim3(256), 0,
                       stream, y, thr, rows, c_out, (c_out + 31) / 32, y_packed);
    return hipGetLastError();
}

}  // namespace bcnn
