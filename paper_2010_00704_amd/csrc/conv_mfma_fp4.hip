// Binary convolution on the matrix cores.
//
// +-1 is exactly representable in the 4-bit float format E2M1 (+1.0 = 0b0010,
// -1.0 = 0b1010), products of +-1 are +-1 and fp32 sums of fewer than 2^24 of
// them are exact, so v_mfma_f32_32x32x64_f8f6f4 with both operands in fp4
// computes the same integer as K - 2*popcount(x xor w) (BCNN paper, Section 1:
// the operator is a matrix product; Section 4.2.1: operands are +-1) at 8x the
// rate of the xor/popcount path on the vector ALUs.
//
// Operands stay 1 bit per element in HBM, L2 and LDS.  A lane expands one
// packed 32-bit word (32 consecutive K positions of its row) into the four
// VGPRs of an fp4 fragment right before the MFMA, with 7 vector ops:
//     frag[j] = ((word << (3-j)) & 0x88888888) | 0x22222222,  j = 0..3
// i.e. bit b of the word becomes the sign bit of some nibble and every nibble
// has magnitude 1.  Which nibble a bit lands in does not matter: both operands
// use the same mapping and the sum over K is order independent.  A set bit
// (+1) becomes -1.0 on BOTH sides, so every product is unchanged.  Positions
// that are 0 in both operands (channel tail bits, zero-filled K padding)
// contribute +1 each; their count Z is known on the host and is folded into
// the accumulator's initial value.  Out-of-image taps are all-zero words on
// the input side only (= -1 in every channel), exactly the padding convention.
//
// Tiling.  MFMA rows (M of the instruction) are output channels, columns are
// output pixels.  A workgroup of 4 waves (2 x 2) owns 128 channels x 256
// pixels; a wave owns 2 x 4 blocks of 32 x 32 (128 accumulator registers).
// K is walked in chunks of 8 packed words (256 bits = 4 MFMA K-steps) over the
// flattened (tap, channel-word) axis; each chunk of both operands is staged
// once per workgroup in LDS (12 KB, double buffered) with full-width global
// loads, and every wave reads its six fragments' words with one ds_read_b128
// each.  Per chunk a wave issues 32 MFMAs (32 cycles each) and 24 x 7
// expansion ops that run in the MFMAs' shadow.
//
// Epilogue.  Weight rows are permuted inside each 32-channel block so that a
// lane ends up holding 16 CONSECUTIVE channels of one pixel (lane half h,
// register r <-> channel 16h + r).  int32 sums: convert and store 64 B runs.
// Fused sign-pack: the accumulator starts at 0.5 - (Z + thr[channel]), so the
// final value is sum - thr + 0.5, never zero, and its sign bit is the
// complement of the output bit; 16 v_alignbit ops collect the sign bits of a
// block, one cross-half exchange completes the 32-bit word.
#include "bcnn_common.h"

namespace bcnn {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int WG_CH = 128;      // channels per workgroup
constexpr int WG_PX = 256;      // pixels per workgroup
constexpr int CB = 2;           // channel blocks per wave
constexpr int PB = 4;           // pixel blocks per wave
constexpr int A_UNITS = WG_CH * 2;  // 16-byte units per stage, weights
constexpr int B_UNITS = WG_PX * 2;  //                         inputs
constexpr int STAGE_UNITS = A_UNITS + B_UNITS;

// MFMA row i of a 32-row block carries this channel of the block (see header).
__device__ __forceinline__ int row_to_channel(int i)
{
    return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
}

// The two masks live in VGPRs (the asm hides their values from the optimiser)
// so that (x & m8) | c2 is one v_and_or_b32; as literals they would force the
// two-instruction VOP2 form, because VOP3 encodings take no literal here.
struct Fp4Masks { uint32_t m8, c2; };
__device__ __forceinline__ Fp4Masks fp4_masks()
{
    Fp4Masks k;
    asm volatile("v_mov_b32 %0, 0x88888888" : "=v"(k.m8));
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(k.c2));
    return k;
}

__device__ __forceinline__ v8i expand_fp4(uint32_t word, const Fp4Masks& k)
{
    v8i f = {0, 0, 0, 0, 0, 0, 0, 0};
    f[0] = (int)(((word << 3) & k.m8) | k.c2);
    f[1] = (int)(((word << 2) & k.m8) | k.c2);
    f[2] = (int)(((word << 1) & k.m8) | k.c2);
    f[3] = (int)((word & k.m8) | k.c2);
    return f;
}

struct MfmaArgs {
    ConvShape s;
    int32_t n_ptiles, n_ctiles;
    int32_t units_per_tap;  // cw / 4
    int32_t n_units;        // taps * cw / 4: 16-byte units along K that hold real data
    int32_t n_chunks;       // ceil(n_units / 2)
    int32_t z;              // 256 * n_chunks - K: positions that count +1 on their own
};

template <bool FUSED>
__global__ __launch_bounds__(256, 2) void conv_mfma_fp4_kernel(
    MfmaArgs a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out)
{
    __shared__ uint4 stage[2][STAGE_UNITS];
    const ConvShape& s = a.s;
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wc = wave & 1, wp = wave >> 1;

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs; give
    // each XCD a contiguous range of tiles (channel tile fastest) so that the
    // workgroups sharing an input tile share an L2.
    int tile = blockIdx.x;
    const int n_tiles = a.n_ptiles * a.n_ctiles;
    const int per_xcd = n_tiles >> 3;
    if (tile < per_xcd * 8) tile = (tile & 7) * per_xcd + (tile >> 3);
    const int ctile = tile % a.n_ctiles;
    const int ptile = tile / a.n_ctiles;
    const int o0 = ctile * WG_CH;
    const int m0 = ptile * WG_PX;

    // ---- loader state: this thread stages one weight unit and two input units per chunk
    const int half = t & 1;
    const int lrow = t >> 1;  // 0..127
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

    // Position of the next chunk's two 16-byte K-units (even unit: half 0, odd
    // unit: half 1) as (filter row u, filter column v, unit within the tap).
    // Wave-uniform and advanced incrementally, so no integer division runs in
    // the loop; a thread picks the entry of its half.
    struct KPos { int u, v, ut; };
    auto advance = [&](KPos& p) {
        if (++p.ut == a.units_per_tap) {
            p.ut = 0;
            if (++p.v == s.ks) { p.v = 0; ++p.u; }
        }
    };
    KPos k0 = {0, 0, 0}, k1 = {0, 0, 0};
    advance(k1);

    uint4 ga, gb[2];
    auto fetch = [&](int chunk) {  // must be called with chunk = 0, 1, 2, ... in order
        const int uu = chunk * 2 + half;  // this thread's unit along K
        const bool real = uu < a.n_units;
        ga = real ? *reinterpret_cast<const uint4*>(wsrc + (size_t)uu * 4) : make_uint4(0, 0, 0, 0);
        const int u = half ? k1.u : k0.u;
        const int v = half ? k1.v : k0.v;
        const int off = (half ? k1.ut : k0.ut) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ih = ph[i] + u, iw = pw[i] + v;
            const bool ok = real && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            const int ihc = ok ? ih : 0, iwc = ok ? iw : 0;
            const uint32_t* p = x + ((size_t)(pn[i] * s.h + ihc) * s.w + iwc) * s.cw + off;
            gb[i] = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
        }
        advance(k0); advance(k0);
        advance(k1); advance(k1);
    };
    auto commit = [&](int buf) {
        stage[buf][a_slot] = ga;
        stage[buf][b_slot[0]] = gb[0];
        stage[buf][b_slot[1]] = gb[1];
    };

    // ---- accumulators: lane (pixel j = lane%32, half h = lane/32), register r
    //      <-> channel 32*block + 16h + r
    v16f acc[CB][PB];
    const int hsel = lane >> 5;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        float init[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v0 = -(float)a.z;
            if constexpr (FUSED) {
                int ch = o0 + 64 * wc + 32 * cb + 16 * hsel + r;
                ch = ch < s.c_out ? ch : s.c_out - 1;
                int th = thr[ch];
                // |y| <= K, so thresholds beyond +-(K+1) decide nothing new
                th = th > s.k + 1 ? s.k + 1 : (th < -s.k - 1 ? -s.k - 1 : th);
                v0 = 0.5f - (float)(a.z + th);  // exact: multiples of 0.5 below 2^23
            }
            init[r] = v0;
        }
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = init[r];
    }

    const Fp4Masks masks = fp4_masks();
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
        for (int ks = 0; ks < 4; ++ks) {
            v8i fa[CB], fb[PB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const uint32_t wd = ks == 0 ? ua[cb].x : ks == 1 ? ua[cb].y : ks == 2 ? ua[cb].z : ua[cb].w;
                fa[cb] = expand_fp4(wd, masks);
            }
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const uint32_t wd = ks == 0 ? ub[pb].x : ks == 1 ? ub[pb].y : ks == 2 ? ub[pb].z : ub[pb].w;
                fb[pb] = expand_fp4(wd, masks);
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    acc[cb][pb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[cb], fb[pb], acc[cb][pb], 4 /*A: fp4*/, 4 /*B: fp4*/, 0, 0, 0, 0);
        }

        if (more) commit(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue
    const int j = lane & 31;
    if constexpr (FUSED) {
        uint32_t* yp = static_cast<uint32_t*>(out);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            uint32_t part[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                uint32_t sg = 0;
#pragma unroll
                for (int r = 15; r >= 0; --r)  // r = 0 ends in bit 0
                    sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(acc[cb][pb][r]), 31);
                part[cb] = ~sg & 0xFFFFu;     // bit r = (sum >= thr) for channel 16h + r
            }
            // lanes of half 0 finish block 0, lanes of half 1 finish block 1
            const uint32_t give = hsel ? part[0] : part[1];
            const uint32_t got = (uint32_t)__shfl_xor((int)give, 32, 64);
            const uint32_t mine = hsel ? part[1] : part[0];
            uint32_t word = hsel ? (got | (mine << 16)) : (mine | (got << 16));
            const int m = m0 + 128 * wp + 32 * pb + j;
            const int wi = (o0 >> 5) + 2 * wc + hsel;  // packed word index along channels
            if (m < s.m && wi < s.cwo) {
                const int valid = s.c_out - 32 * wi;   // real channels in this word
                if (valid < 32) word &= (1u << valid) - 1u;
                yp[(size_t)m * s.cwo + wi] = word;
            }
        }
    } else {
        int32_t* y = static_cast<int32_t*>(out);
        const bool vec_ok = (s.c_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) & 15) == 0);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int m = m0 + 128 * wp + 32 * pb + j;
            if (m >= s.m) continue;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int c0 = o0 + 64 * wc + 32 * cb + 16 * hsel;
                int32_t* row = y + (size_t)m * s.c_out + c0;
                if (vec_ok && c0 + 16 <= s.c_out) {
#pragma unroll
                    for (int r = 0; r < 16; r += 4) {
                        int4 q;
                        q.x = (int)acc[cb][pb][r + 0];
                        q.y = (int)acc[cb][pb][r + 1];
                        q.z = (int)acc[cb][pb][r + 2];
                        q.w = (int)acc[cb][pb][r + 3];
                        *reinterpret_cast<int4*>(row + r) = q;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (c0 + r < s.c_out) row[r] = (int)acc[cb][pb][r];
                }
            }
        }
    }
}

}  // namespace

bool conv_mfma_fp4_supported(const ConvShape& s, const uint32_t* x, const uint32_t* w)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w);
    const int64_t n_units = (int64_t)s.ks * s.ks * s.cw / 4;
    const int64_t n_chunks = (n_units + 1) / 2;
    // 16-byte units must not straddle taps; every partial sum (a multiple of
    // 0.5 in the fused case) must be exact in fp32
    return s.cw % 4 == 0 && (bits & 15) == 0 && 256 * n_chunks + s.k + 2 < (1 << 22);
}

hipError_t launch_conv_mfma_fp4(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                                const int32_t* thr, void* out, hipStream_t stream)
{
    MfmaArgs a;
    a.s = s;
    a.n_ptiles = (s.m + WG_PX - 1) / WG_PX;
    a.n_ctiles = (s.c_out + WG_CH - 1) / WG_CH;
    a.units_per_tap = s.cw / 4;
    a.n_units = s.ks * s.ks * a.units_per_tap;
    a.n_chunks = (a.n_units + 1) / 2;
    a.z = 256 * a.n_chunks - s.k;
    const unsigned blocks = (unsigned)(a.n_ptiles * a.n_ctiles);
    if (thr)
        hipLaunchKernelGGL(conv_mfma_fp4_kernel<true>, dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out);
    else
        hipLaunchKernelGGL(conv_mfma_fp4_kernel<false>, dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out);
    return hipGetLastError();
}

}  // namespace bcnn
