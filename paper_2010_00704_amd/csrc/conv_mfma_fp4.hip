// Binary convolution on the matrix cores.
//
// +-1 is exactly representable in the 4-bit float format E2M1 (+1.0 = 0b0010,
// -1.0 = 0b1010; the other codes used below are 0.5, 2, 4 and 0), products
// are small integers and fp32 sums of fewer than 2^22 of them are exact, so v_mfma_f32_32x32x64_f8f6f4 with both operands in fp4
// computes the same integer as K - 2*popcount(x xor w) (BCNN paper, Section 1:
// the operator is a matrix product; Section 4.2.1: operands are +-1) at 8x the
// rate of the xor/popcount path on the vector ALUs.
//
// Operands stay 1 bit per element in HBM, L2 and LDS.  A lane expands one
// packed 32-bit word (32 consecutive K positions of its row) into the four
// VGPRs of an fp4 fragment right before the MFMA.  VGPR j of a fragment takes
// the bits 4i+j of the word on both sides (the sum over K is order
// independent, only the pairing matters).  Vector-ALU work per MFMA is the
// limit here (about four vector ops hide under one 32-cycle MFMA, measured),
// so the side with many fragments, the inputs, gets the cheapest expansion:
//     j = 3 : (word & 0x88888888) | 0x22222222   sign bit over magnitude 1
//     j < 3 :  word & (0x11111111 << j)          the bit alone: 0 or 0.5/1/2
// 4 ops per fragment, no shifts.  The weights (few fragments) compensate:
//     j = 3 : as above
//     j < 3 : ((~word << (3-j)) & 0x88888888) | magnitude 4/2/1
// 8 ops.  With s = +-1 the value of a bit: j = 3 gives (-s_w)(-s_x) = s_w*s_x;
// j < 3 gives (alpha*s_w)(beta*bit_x) = s_w*(1 + s_x) = s_w + s_w*s_x.  So the
// MFMA sum is the wanted dot product plus, per output channel, the sum of
// that channel's weights over the positions 4i+0..2 = 2*pop - 24*words.  The
// threads that stream the weights into LDS count pop on the way, and the
// epilogue subtracts it.  All partial sums are integers (or multiples of 0.5
// in the fused case) below 2^23: exact in fp32.  Positions that are 0 in both
// operands (channel tail bits, zero-filled K padding) contribute +1 at j = 3
// and 0 at j < 3; the host folds their count into the accumulator's initial
// value.  Out-of-image taps are all-zero words on the input side only (= -1 in
// every channel), exactly the padding convention.
//
// Tiling.  MFMA rows (M of the instruction) are output channels, columns are
// output pixels.  A workgroup of 4 waves (2 x 2) owns 128 channels x 64*PB
// pixels; a wave owns 2 x PB blocks of 32 x 32 (PB = 4 or 7; 7 divides the
// pixel counts of 7/14/28/56-wide feature maps, see the launcher).
// K is walked in chunks of 8 packed words (256 bits = 4 MFMA K-steps) over the
// flattened (tap, channel-word) axis; each chunk of both operands is staged
// once per workgroup in LDS (double buffered) with full-width global loads,
// and every wave reads each fragment's words with one ds_read_b128.  Per
// chunk a wave issues 8*PB MFMAs (32 cycles each) and 4*(2+PB)*7 expansion
// ops; only about 3 vector ops per MFMA hide in its shadow (measured), which
// is why the wide tile matters.
//
// Epilogue.  Weight rows are permuted inside each 32-channel block so that a
// lane ends up holding 16 CONSECUTIVE channels of one pixel (lane half h,
// register r <-> channel 16h + r).  int32 sums: subtract the per-channel
// constant, convert and store 64 B runs.  Fused sign-pack: subtract constant
// + thr[channel] - 0.5, so the value is sum - thr + 0.5, never zero, and its
// sign bit is the complement of the output bit; 16 v_alignbit ops collect the
// sign bits of a block, one cross-half exchange completes the 32-bit word.
#include "bcnn_common.h"

#include <utility>

namespace bcnn {
namespace {

// Compile-time loop: f(std::integral_constant<int, 0>) ... f(<N-1>), so that
// every index inside is a constant expression.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int WG_CH = 128;  // channels per workgroup (2 waves x 2 blocks of 32)
constexpr int CB = 2;       // channel blocks per wave

// MFMA row i of a 32-row block carries this channel of the block (see header).
__device__ __forceinline__ int row_to_channel(int i)
{
    return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
}

// Constants that enter v_and_or_b32 live in VGPRs (the asm hides their values
// from the optimiser): as literals they would force the two-instruction VOP2
// form, because VOP3 encodings take no literal here.
struct Fp4Masks { uint32_t m8, c2, c4, c6; };
__device__ __forceinline__ Fp4Masks fp4_masks()
{
    Fp4Masks k;
    asm volatile("v_mov_b32 %0, 0x88888888" : "=v"(k.m8));
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(k.c2));
    asm volatile("v_mov_b32 %0, 0x44444444" : "=v"(k.c4));
    asm volatile("v_mov_b32 %0, 0x66666666" : "=v"(k.c6));
    return k;
}

__device__ __forceinline__ uint32_t pick(const uint4& q, int i)
{
    return i == 0 ? q.x : i == 1 ? q.y : i == 2 ? q.z : q.w;
}

struct MfmaArgs {
    ConvShape s;
    int32_t n_ptiles, n_ctiles;
    int32_t units_per_tap;  // cw / 4
    int32_t n_units;        // taps * cw / 4: 16-byte units along K that hold real data
    int32_t n_chunks;       // ceil(n_units / 2)
    int32_t z;              // 256 * n_chunks - K: positions that count +1 on their own
    int32_t x_bytes, w_bytes;  // sizes of the packed tensors, for the buffer descriptors
};

// PB = pixel blocks (of 32) per wave; the workgroup covers 2*32*PB pixels.
template <int PB, bool FUSED>
__global__ __launch_bounds__(256, (PB <= 4 ? 2 : 1)) void conv_mfma_fp4_kernel(
    MfmaArgs a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out)
{
    constexpr int WG_PX = 64 * PB;
    constexpr int B_UNITS = WG_PX * 2;
    constexpr int NB = (B_UNITS + 255) / 256;  // input units staged per thread and chunk
    // One stage = the chunk's 8 K-words of every row, as 8-byte elements
    // [K-half][word pair][row]: a lane reads the pair it needs with one
    // ds_read_b64, lanes of a half-wave at consecutive addresses.
    constexpr int A_ELEMS = 4 * WG_CH, B_ELEMS = 4 * WG_PX;
    constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
    __shared__ uint2 stage[2][STAGE_ELEMS + 1];  // + 1: spare element for out-of-tile rows
    __shared__ int wpop_lds[WG_CH];
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

    // ---- loader state.  Per chunk a thread stages one 16-byte weight unit and
    // up to NB input units; its K-half (even or odd unit of the chunk) is fixed.
    const int half = t & 1;
    const int lrow = t >> 1;  // 0..127
    int wrow_bytes;
    {
        int ch = o0 + 32 * (lrow >> 5) + row_to_channel(lrow & 31);
        ch = ch < s.c_out ? ch : s.c_out - 1;
        wrow_bytes = ch * a.n_units * 16;
    }
    const int a_slot = half * 2 * WG_CH + lrow;   // element of word pair 0; pair 1 is WG_CH further
    // For input row i: word offset of the window's top-left tap (may point
    // outside the image; only used where the tap's validity bit is set) and
    // one validity bit per tap.
    int rbase[NB];
    uint32_t vmask[NB];
    int b_slot[NB];
    int b_pair1 = WG_PX;     // distance from a row's word pair 0 to its pair 1 (0: both go to the spare element)
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int row = lrow + 128 * i;
        const bool row_ok = row < WG_PX;
        int m = m0 + (row_ok ? row : 0);
        m = m < s.m ? m : s.m - 1;
        const int hw = s.ho * s.wo;
        const int n = m / hw;
        const int r = m - n * hw;
        const int oh = r / s.wo;
        const int ph = oh * s.stride - s.pad;
        const int pw = (r - oh * s.wo) * s.stride - s.pad;
        rbase[i] = ((n * s.h + ph) * s.w + pw) * s.cw;
        uint32_t vm = 0;
        for (int u = 0; u < s.ks; ++u)
            for (int v = 0; v < s.ks; ++v) {
                const int ih = ph + u, iw = pw + v;
                if (row_ok && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w) vm |= 1u << (u * s.ks + v);
            }
        vmask[i] = vm;
        b_slot[i] = row_ok ? A_ELEMS + half * 2 * WG_PX + row : STAGE_ELEMS;
        if (i == NB - 1) b_pair1 = row_ok ? WG_PX : 0;   // only the last row of a thread can be out of the tile
    }

    // Position of this thread's next K-unit (even units for half 0, odd for
    // half 1): tap index, filter column, unit within the tap, and the word
    // offset relative to the window's top-left tap.  Advanced one unit at a
    // time with selects only (per-thread values, so the compiler keeps them
    // on the vector ALU and the loop body stays free of branches); no
    // division runs in the loop.
    const int row_jump = (s.w - s.ks) * s.cw;
    int f_unit = 0, f_tap = 0, f_v = 0, f_ut = 0, f_off = 0;
    auto advance = [&]() {
        const int ut1 = f_ut + 1;
        const bool tap_done = ut1 == a.units_per_tap;
        f_ut = tap_done ? 0 : ut1;
        f_tap += tap_done ? 1 : 0;
        const int v1 = f_v + (tap_done ? 1 : 0);
        const bool row_done = v1 == s.ks;
        f_v = row_done ? 0 : v1;
        f_off += 4 + (row_done ? row_jump : 0);
        f_unit += 1;
    };
    if (half) advance();

    // Global -> registers, one 16-byte unit per call.  Raw buffer loads: a
    // lane whose unit must read as zero (out-of-image tap, K padding past the
    // last real unit) gets an offset beyond the buffer and the hardware range
    // check returns 0, so the loader has no branches.
    const __amdgpu_buffer_rsrc_t xres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(x), 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t wres =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(w), 0, a.w_bytes, 0x00020000);
    constexpr uint32_t OOB = 0xFFFFFFF0u;
    v4i ga, gb[NB];
    int wpop = 0;            // set weight bits at positions 4i+0..2 seen by this thread
    // (Offsets are chosen with mask arithmetic, not ?:, which the compiler
    // would turn into divergent branches that split the loop body.)
    auto fetch_piece = [&](int j) {  // j = 0: weights; j = 1..NB: input rows
        const uint32_t real = f_unit < a.n_units ? 1u : 0u;
        if (j == 0) {
            const uint32_t m = 0u - real;
            const uint32_t o = ((uint32_t)(wrow_bytes + f_unit * 16) & m) | (OOB & ~m);
            ga = __builtin_amdgcn_raw_buffer_load_b128(wres, o, 0, 0);
        } else {
            const int i = j - 1;
            const uint32_t m = 0u - (real & (vmask[i] >> (f_tap & 31)));
            const uint32_t o = (((uint32_t)(rbase[i] + f_off) << 2) & m) | (OOB & ~m);
            gb[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, o, 0, 0);
        }
    };
    // Threads whose input row lies beyond the tile write to the spare element
    // behind the stage instead of branching around the store.
    auto commit_piece = [&](int buf, int j) {
        uint2* st = stage[buf];
        if (j == 0) {
            st[a_slot] = make_uint2((uint32_t)ga[0], (uint32_t)ga[1]);
            st[a_slot + WG_CH] = make_uint2((uint32_t)ga[2], (uint32_t)ga[3]);
            wpop += __builtin_popcount((uint32_t)ga[0] & 0x77777777u) + __builtin_popcount((uint32_t)ga[1] & 0x77777777u) +
                    __builtin_popcount((uint32_t)ga[2] & 0x77777777u) + __builtin_popcount((uint32_t)ga[3] & 0x77777777u);
        } else {
            st[b_slot[j - 1]] = make_uint2((uint32_t)gb[j - 1][0], (uint32_t)gb[j - 1][1]);
            st[b_slot[j - 1] + (j == NB ? b_pair1 : WG_PX)] = make_uint2((uint32_t)gb[j - 1][2], (uint32_t)gb[j - 1][3]);
        }
    };

    // ---- accumulators: lane (pixel j = lane%32, half h = lane/32), register r
    //      <-> channel 32*block + 16h + r.  They start at zero; every constant
    //      and per-channel term is applied in the epilogue.
    v16f acc[CB][PB];
    const int hsel = lane >> 5;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;

    // ---- main loop, software pipelined by hand.
    // A wave issues in order, so whatever follows a run of MFMAs in program
    // order waits for all of them to issue; only work placed BETWEEN MFMAs
    // overlaps with the matrix core.  Each chunk is therefore a fixed program
    // of 4 K-steps x PB pixel blocks x 2 channel blocks MFMA slots, and after
    // every MFMA comes a small piece of the other work (order pinned by
    // scheduling barriers):
    //   every slot : half of an input fragment two blocks ahead (fragments
    //                live in a ring of four, so few registers hold them) and
    //                a share of the next K-step's two weight fragments
    //   K-step 0   : LDS commit of chunk c+1 (global loads issued one chunk
    //                earlier) and LDS reads of this chunk's second word pair;
    //                workgroup barrier at the end of the step
    //   K-step 1   : global loads of chunk c+2
    //   K-step 2   : LDS reads of chunk c+1's first word pair
    //   K-step 3   : loader bookkeeping
    // Buffer c%2 is last read in K-step 0 of chunk c (before that chunk's
    // barrier) and next written in K-step 0 of chunk c+1 (after it).
    constexpr int NF = CB + PB;       // words per lane and K-step: weights first, then inputs
    constexpr int NS = CB * PB;       // MFMA slots per K-step
    static_assert(CB == 2, "slot program assumes two channel blocks");
    static_assert(NB + 1 <= NS && NF <= NS, "side work must fit the MFMA slots of a K-step");
    const Fp4Masks masks = fp4_masks();
    int fa[2][CB][4];                 // weight fragments, double buffered over K-steps
    int fb[4][4];                     // input fragments, ring over (K-step, pixel block)
    uint2 p0[NF], p1[NF];             // this lane's words of K-steps 0,1 and 2,3 of the chunk
    auto read_pair = [&](uint2 (&dst)[NF], int buf, int kp, int f) {
        const int e = f < CB ? (hsel * 2 + kp) * WG_CH + 32 * (2 * wc + f) + (lane & 31)
                             : A_ELEMS + (hsel * 2 + kp) * WG_PX + 32 * (PB * wp + (f - CB)) + (lane & 31);
        dst[f] = stage[buf][e];
    };
    auto word_of = [&](int f, int ks) -> uint32_t {   // ks = 0..3 within the chunk
        return ks == 0 ? p0[f].x : ks == 1 ? p0[f].y : ks == 2 ? p1[f].x : p1[f].y;
    };
    // One VGPR (8 nibbles) of a fragment; VGPR jj takes the bits 4i+jj of the
    // packed word on both sides (see the header for the values).
    auto expand_w = [&](uint32_t word, int jj) -> int {
        if (jj == 3) return (int)((word & masks.m8) | masks.c2);
        return (int)(((~word << (3 - jj)) & masks.m8) | (jj == 0 ? masks.c6 : jj == 1 ? masks.c4 : masks.c2));
    };
    auto expand_x = [&](uint32_t word, int jj) -> int {
        if (jj == 3) return (int)((word & masks.m8) | masks.c2);
        return (int)(word & (0x11111111u << jj));
    };
    auto mfma_one = [&](int ks, int cb, int pb) {
        const int (&A)[4] = fa[ks & 1][cb];
        const int (&Bf)[4] = fb[(ks * PB + pb) & 3];
        const v8i va = {A[0], A[1], A[2], A[3], 0, 0, 0, 0};
        const v8i vb = {Bf[0], Bf[1], Bf[2], Bf[3], 0, 0, 0, 0};
        acc[cb][pb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
            va, vb, acc[cb][pb], 4 /*A: fp4*/, 4 /*B: fp4*/, 0, 0, 0, 0);
    };
    // One chunk.  On entry p0 holds its first word pair, fa[0] its K-step 0
    // weight fragments and fb[0], fb[1] its first two input fragments; on exit
    // the same holds for the next chunk.  nbuf = stage buffer of chunk c+1.
    auto chunk_body = [&](int nbuf) {
        static_for<4 * NS>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int ks = i / NS, sl = i % NS;   // K-step, slot within it
            constexpr int pb = sl / CB, cb = sl % CB;
            mfma_one(ks, cb, pb);
            // input fragment two blocks ahead: registers 2*cb, 2*cb+1.  Past the
            // end of the chunk this reads p0 of the next chunk (loaded in K-step 2).
            {
                constexpr int q = ks * PB + pb + 2;           // linear (K-step, block) index
                constexpr int qks = (q / PB) & 3, qpb = q % PB;
                const uint32_t word = word_of(CB + qpb, qks);
                fb[q & 3][2 * cb] = expand_x(word, 2 * cb);
                fb[q & 3][2 * cb + 1] = expand_x(word, 2 * cb + 1);
            }
            // next K-step's weight fragments: 8 registers over the NS slots
            static_for<(sl + 1) * 8 / NS - sl * 8 / NS>([&](auto jc) {
                constexpr int idx = sl * 8 / NS + decltype(jc)::value;
                constexpr int f = idx >> 2, jj = idx & 3;
                fa[(ks + 1) & 1][f][jj] = expand_w(word_of(f, (ks + 1) & 3), jj);
            });
            // side work, spread over the slots of its K-step
            if constexpr (ks == 0) {
                constexpr int NP = 1 + NB + NF;               // commits, then reads of pair 1
                static_for<NP>([&](auto pc) {
                    constexpr int pidx = decltype(pc)::value;
                    if constexpr (pidx * NS / NP == sl) {
                        if constexpr (pidx <= NB) commit_piece(nbuf, pidx);
                        else read_pair(p1, nbuf ^ 1, 1, pidx - 1 - NB);
                    }
                });
                if constexpr (sl == NS - 1) __syncthreads();
            }
            if constexpr (ks == 1 && sl <= NB) fetch_piece(sl);
            if constexpr (ks == 2 && sl < NF) read_pair(p0, nbuf, 0, sl);
            if constexpr (ks == 3 && sl < 2) advance();       // on to the unit of the next fetch
            __builtin_amdgcn_sched_barrier(0);
        });
    };

#pragma unroll
    for (int j = 0; j <= NB; ++j) fetch_piece(j);
#pragma unroll
    for (int j = 0; j <= NB; ++j) commit_piece(0, j);
    advance(); advance();
#pragma unroll
    for (int j = 0; j <= NB; ++j) fetch_piece(j);   // chunk 1, committed during chunk 0
    advance(); advance();
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) read_pair(p0, 0, 0, f);
#pragma unroll
    for (int f = 0; f < CB; ++f)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) fa[0][f][jj] = expand_w(p0[f].x, jj);
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) fb[q][jj] = expand_x(p0[CB + q].x, jj);

    for (int chunk = 0; chunk < a.n_chunks; ++chunk) chunk_body((chunk + 1) & 1);

    // ---- epilogue
    // The accumulator holds  sum + Z - 192*n_chunks + 2*pop(channel)  (Z:
    // positions that are zero on both sides and count +1, see the launcher;
    // pop: the channel's set weight bits at positions 4i+0..2, see the
    // header).  The two threads that streamed a weight row add their counts
    // and the workgroup exchanges them through LDS indexed by channel.  What
    // has to be subtracted per channel (plus the threshold, minus 0.5 so that
    // the result is never zero, in the fused case) is kept in sub[][].
    float sub[CB][16];
    {
        const int both = wpop + __shfl_xor(wpop, 1, 64);
        if (half == 0) wpop_lds[32 * (lrow >> 5) + row_to_channel(lrow & 31)] = both;
        __syncthreads();
        const int base = a.z - 192 * a.n_chunks;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cl = 64 * wc + 32 * cb + 16 * hsel + r;
                int v = base + 2 * wpop_lds[cl];
                if constexpr (FUSED) {
                    int ch = o0 + cl;
                    ch = ch < s.c_out ? ch : s.c_out - 1;
                    int th = thr[ch];
                    // |y| <= K, so thresholds beyond +-(K+1) decide nothing new
                    th = th > s.k + 1 ? s.k + 1 : (th < -s.k - 1 ? -s.k - 1 : th);
                    sub[cb][r] = (float)(v + th) - 0.5f;  // exact: multiples of 0.5 below 2^23
                } else {
                    sub[cb][r] = (float)v;
                }
            }
    }
    const int j = lane & 31;
    if constexpr (FUSED) {
        // bit = (y >= thr)  <=>  acc - sub = y - thr + 0.5 > 0  <=>  sign bit clear
        uint32_t* yp = static_cast<uint32_t*>(out);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            uint32_t part[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                uint32_t sg = 0;
#pragma unroll
                for (int r = 15; r >= 0; --r)  // r = 0 ends in bit 0
                    sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(acc[cb][pb][r] - sub[cb][r]), 31);
                part[cb] = ~sg & 0xFFFFu;     // bit r = (sum >= thr) for channel 16h + r
            }
            // lanes of half 0 finish block 0, lanes of half 1 finish block 1
            const uint32_t give = hsel ? part[0] : part[1];
            const uint32_t got = (uint32_t)__shfl_xor((int)give, 32, 64);
            const uint32_t mine = hsel ? part[1] : part[0];
            uint32_t word = hsel ? (got | (mine << 16)) : (mine | (got << 16));
            const int m = m0 + 32 * (PB * wp + pb) + j;
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
            const int m = m0 + 32 * (PB * wp + pb) + j;
            if (m >= s.m) continue;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int c0 = o0 + 64 * wc + 32 * cb + 16 * hsel;
                int32_t* row = y + (size_t)m * s.c_out + c0;
                if (vec_ok && c0 + 16 <= s.c_out) {
#pragma unroll
                    for (int r = 0; r < 16; r += 4) {
                        int4 q;
                        q.x = (int)(acc[cb][pb][r + 0] - sub[cb][r + 0]);
                        q.y = (int)(acc[cb][pb][r + 1] - sub[cb][r + 1]);
                        q.z = (int)(acc[cb][pb][r + 2] - sub[cb][r + 2]);
                        q.w = (int)(acc[cb][pb][r + 3] - sub[cb][r + 3]);
                        *reinterpret_cast<int4*>(row + r) = q;
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (c0 + r < s.c_out) row[r] = (int)(acc[cb][pb][r] - sub[cb][r]);
                }
            }
        }
    }
}

template <int PB, bool FUSED>
hipError_t launch_pb(MfmaArgs a, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                     void* out, hipStream_t stream)
{
    constexpr int WG_PX = 64 * PB;
    a.n_ptiles = (a.s.m + WG_PX - 1) / WG_PX;
    const unsigned blocks = (unsigned)(a.n_ptiles * a.n_ctiles);
    hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, FUSED>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out);
    return hipGetLastError();
}

}  // namespace

bool conv_mfma_fp4_supported(const ConvShape& s, const uint32_t* x, const uint32_t* w)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w);
    const int64_t n_units = (int64_t)s.ks * s.ks * s.cw / 4;
    const int64_t n_chunks = (n_units + 1) / 2;
    // 16-byte units must not straddle taps; every partial sum (a multiple of
    // 0.5 in the fused case) must be exact in fp32
    // and both packed tensors must be addressable by 31-bit byte offsets
    const int64_t x_bytes = (int64_t)s.n * s.h * s.w * s.cw * 4;
    const int64_t w_bytes = (int64_t)s.c_out * n_units * 16;
    return s.cw % 4 == 0 && (bits & 15) == 0 && 256 * n_chunks + s.k + 2 < (1 << 22) &&
           x_bytes < (1ll << 31) && w_bytes < (1ll << 31);
}

// Rounds of workgroups over the 256 CUs times the work of one workgroup:
// the time a tile width costs if every workgroup ran at the same rate.
static double tile_cost(const ConvShape& s, int pb)
{
    const int64_t wg_px = 64 * pb;
    const int64_t wgs = ((s.m + wg_px - 1) / wg_px) * ((s.c_out + WG_CH - 1) / WG_CH);
    const int64_t rounds = (wgs + 255) / 256;
    return (double)rounds * pb;
}

hipError_t launch_conv_mfma_fp4(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                                const int32_t* thr, void* out, hipStream_t stream)
{
    MfmaArgs a;
    a.s = s;
    a.n_ptiles = 0;  // set by launch_pb
    a.n_ctiles = (s.c_out + WG_CH - 1) / WG_CH;
    a.units_per_tap = s.cw / 4;
    a.n_units = s.ks * s.ks * a.units_per_tap;
    a.n_chunks = (a.n_units + 1) / 2;
    a.z = 256 * a.n_chunks - s.k;
    a.x_bytes = (int32_t)((int64_t)s.n * s.h * s.w * s.cw * 4);
    a.w_bytes = (int32_t)((int64_t)s.c_out * a.n_units * 16);
    // Feature maps of 7, 14, 28, 56 pixels a side make the pixel count a
    // multiple of 49: 7 pixel blocks per wave then tile it without remainder
    // where 4 would leave a quarter of the last round idle.
    // (Only the fused kernel has the registers for it: the int32 epilogue of
    // a 2 x 7 tile would spill.)
    if (!thr) return launch_pb<4, false>(a, x, w, thr, out, stream);
    if (tile_cost(s, 7) < tile_cost(s, 4)) return launch_pb<7, true>(a, x, w, thr, out, stream);
    return launch_pb<4, true>(a, x, w, thr, out, stream);
}

}  // namespace bcnn
