// Binary convolution on the matrix cores with int8 operands: the benchmark arm
// that the fp4 kernel (conv_mfma_fp4.hip) is measured against.
//
// Every packed bit is expanded to one int8 (+1 = 0x01, -1 = 0xFF) in registers
// and v_mfma_i32_32x32x32_i8 sums the products exactly in int32 (BCNN paper,
// Section 1: the operator is a matrix product; Section 4.2.1: operands are
// +-1).  Against fp4 this format has half the matrix rate and needs four
// vector ops per 4 elements (bit-field extract, multiply-spread, mask, byte
// lookup) instead of one op per 8, so it is vector-ALU bound; it is kept as a
// selectable variant for measurement only and AUTO never picks it.
//
// Structure (deliberately plain): workgroup of 4 waves (2 x 2) = 128 channels
// x 256 pixels, a wave owns 2 x 4 blocks of 32 x 32.  K is walked in chunks
// of 8 packed words; each thread stages 16-byte units of both operands through
// registers into LDS (double buffered, one barrier per chunk); a lane reads
// its row's 128 bits per block with one ds_read_b128 and feeds eight MFMA
// K-steps of 16 bits each from them.  Positions that are 0 in both operands
// (channel tail bits, zero-filled K padding) are (-1)(-1) = +1 each; their
// count Z is subtracted in the epilogue.  The epilogue mirrors the fp4
// kernel's: weight rows permuted so a lane holds 16 consecutive channels.
#include "bcnn_common.h"

namespace bcnn {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WG_CH = 128, WG_PX = 256, CB = 2, PB = 4;
constexpr int A_UNITS = WG_CH * 2, B_UNITS = WG_PX * 2, STAGE_UNITS = A_UNITS + B_UNITS;

__device__ __forceinline__ int row_to_channel(int i)
{
    return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
}

// 16 bits (bits [lo, lo+16) of word) -> 16 int8 in four VGPRs; byte b of VGPR q
// is bit lo + 4q + b: 1 -> 0x01, 0 -> 0xFF.
__device__ __forceinline__ v4i expand_i8(uint32_t word, int lo)
{
    v4i f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t nib = (word >> (lo + 4 * q)) & 0xFu;
        // bit 0 stays, bit 1 -> 8, bit 2 -> 16, bit 3 -> 24
        const uint32_t sel = (nib * 0x00204081u) & 0x01010101u;
        f[q] = (int)__builtin_amdgcn_perm(0u, 0x000001FFu, sel);  // selector byte 0 -> 0xFF, 1 -> 0x01
    }
    return f;
}

struct I8Args {
    ConvShape s;
    int32_t n_ptiles, n_ctiles, units_per_tap, n_units, n_chunks, z;
};

template <bool FUSED>
__global__ __launch_bounds__(256, 2) void conv_mfma_i8_kernel(
    I8Args a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out)
{
    __shared__ uint4 stage[2][STAGE_UNITS];
    const ConvShape& s = a.s;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wc = wave & 1, wp = wave >> 1;
    const int tile = blockIdx.x;
    const int o0 = (tile % a.n_ctiles) * WG_CH;
    const int m0 = (tile / a.n_ctiles) * WG_PX;

    // loader: thread stages one weight unit and two input units per chunk
    const int half = t & 1, lrow = t >> 1;
    const uint32_t* wsrc;
    {
        int ch = o0 + 32 * (lrow >> 5) + row_to_channel(lrow & 31);
        ch = ch < s.c_out ? ch : s.c_out - 1;
        wsrc = w + (size_t)ch * ((size_t)a.n_units * 4);
    }
    const int a_slot = (lrow >> 5) * 64 + half * 32 + (lrow & 31);
    int pn[2], ph[2], pw[2], b_slot[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = lrow + 128 * i;
        int m = m0 + row;
        m = m < s.m ? m : s.m - 1;
        const int hw = s.ho * s.wo;
        pn[i] = m / hw;
        const int r = m - pn[i] * hw;
        const int oh = r / s.wo;
        ph[i] = oh * s.stride - s.pad;
        pw[i] = (r - oh * s.wo) * s.stride - s.pad;
        b_slot[i] = A_UNITS + (row >> 5) * 64 + half * 32 + (row & 31);
    }
    uint4 ga, gb[2];
    auto fetch = [&](int chunk) {
        const int uu = chunk * 2 + half;
        const bool real = uu < a.n_units;
        ga = real ? *reinterpret_cast<const uint4*>(wsrc + (size_t)uu * 4) : make_uint4(0, 0, 0, 0);
        const int uc = real ? uu : 0;
        const int tap = uc / a.units_per_tap;
        const int off = (uc - tap * a.units_per_tap) * 4;
        const int u = tap / s.ks, v = tap - u * s.ks;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ih = ph[i] + u, iw = pw[i] + v;
            const bool ok = real && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            const int ihc = ok ? ih : 0, iwc = ok ? iw : 0;
            const uint32_t* p = x + ((size_t)(pn[i] * s.h + ihc) * s.w + iwc) * s.cw + off;
            gb[i] = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
        }
    };
    auto commit = [&](int buf) {
        stage[buf][a_slot] = ga;
        stage[buf][b_slot[0]] = gb[0];
        stage[buf][b_slot[1]] = gb[1];
    };

    v16i acc[CB][PB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0;

    fetch(0);
    commit(0);
    __syncthreads();
    for (int chunk = 0; chunk < a.n_chunks; ++chunk) {
        const int buf = chunk & 1;
        const bool more = chunk + 1 < a.n_chunks;
        if (more) fetch(chunk + 1);
        uint4 ua[CB], ub[PB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) ua[cb] = stage[buf][(2 * wc + cb) * 64 + lane];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) ub[pb] = stage[buf][A_UNITS + (4 * wp + pb) * 64 + lane];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {   // 16 bits of each lane's 128 per step
            v4i fa[CB], fb[PB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const uint32_t wd = (ks >> 1) == 0 ? ua[cb].x : (ks >> 1) == 1 ? ua[cb].y : (ks >> 1) == 2 ? ua[cb].z : ua[cb].w;
                fa[cb] = expand_i8(wd, 16 * (ks & 1));
            }
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const uint32_t wd = (ks >> 1) == 0 ? ub[pb].x : (ks >> 1) == 1 ? ub[pb].y : (ks >> 1) == 2 ? ub[pb].z : ub[pb].w;
                fb[pb] = expand_i8(wd, 16 * (ks & 1));
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    acc[cb][pb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cb], fb[pb], acc[cb][pb], 0, 0, 0);
        }
        if (more) commit(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane (pixel j = lane%32, half h = lane/32), register r <-> channel 32*block + 16h + r
    const int j = lane & 31, hsel = lane >> 5;
    if constexpr (FUSED) {
        uint32_t* yp = static_cast<uint32_t*>(out);
        int sub[CB][16];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int ch = o0 + 64 * wc + 32 * cb + 16 * hsel + r;
                ch = ch < s.c_out ? ch : s.c_out - 1;
                int th = thr[ch];
                th = th > s.k + 1 ? s.k + 1 : (th < -s.k - 1 ? -s.k - 1 : th);
                sub[cb][r] = a.z + th;
            }
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            uint32_t part[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                uint32_t sg = 0;
#pragma unroll
                for (int r = 15; r >= 0; --r)   // sign of (y - thr): set <=> bit 0
                    sg = __builtin_amdgcn_alignbit(sg, (uint32_t)(acc[cb][pb][r] - sub[cb][r]), 31);
                part[cb] = ~sg & 0xFFFFu;
            }
            const uint32_t give = hsel ? part[0] : part[1];
            const uint32_t got = (uint32_t)__shfl_xor((int)give, 32, 64);
            const uint32_t mine = hsel ? part[1] : part[0];
            uint32_t word = hsel ? (got | (mine << 16)) : (mine | (got << 16));
            const int m = m0 + 128 * wp + 32 * pb + j;
            const int wi = (o0 >> 5) + 2 * wc + hsel;
            if (m < s.m && wi < s.cwo) {
                const int valid = s.c_out - 32 * wi;
                if (valid < 32) word &= (1u << valid) - 1u;
                yp[(size_t)m * s.cwo + wi] = word;
            }
        }
    } else {
        int32_t* y = static_cast<int32_t*>(out);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int m = m0 + 128 * wp + 32 * pb + j;
            if (m >= s.m) continue;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int c0 = o0 + 64 * wc + 32 * cb + 16 * hsel;
                int32_t* row = y + (size_t)m * s.c_out + c0;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (c0 + r < s.c_out) row[r] = acc[cb][pb][r] - a.z;
            }
        }
    }
}

}  // namespace

bool conv_mfma_i8_supported(const ConvShape& s, const uint32_t* x, const uint32_t* w)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w);
    return s.cw % 4 == 0 && (bits & 15) == 0;   // 16-byte units must not straddle taps
}

hipError_t launch_conv_mfma_i8(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                               const int32_t* thr, void* out, hipStream_t stream)
{
    I8Args a;
    a.s = s;
    a.n_ptiles = (s.m + WG_PX - 1) / WG_PX;
    a.n_ctiles = (s.c_out + WG_CH - 1) / WG_CH;
    a.units_per_tap = s.cw / 4;
    a.n_units = s.ks * s.ks * a.units_per_tap;
    a.n_chunks = (a.n_units + 1) / 2;
    a.z = 256 * a.n_chunks - s.k;
    const unsigned blocks = (unsigned)(a.n_ptiles * a.n_ctiles);
    if (thr)
        hipLaunchKernelGGL(conv_mfma_i8_kernel<true>, dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out);
    else
        hipLaunchKernelGGL(conv_mfma_i8_kernel<false>, dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out);
    return hipGetLastError();
}

}  // namespace bcnn
