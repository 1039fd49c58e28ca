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
// pixel counts of 7/14/28/56-wide feature maps, see the launcher).  The tile
// body is a device function (conv_mfma_fp4_tile) shared by two kernels: the
// pixel-major one (GEMM rows = consecutive pixels) and the position-major one
// for small maps in large batches (conv_mfma_fp4_pos_kernel below), which also
// runs it with PB = 5, 6, 8 and with workgroups of 2 waves (2 x 1).
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
#pragma once
#include "bcnn_common.h"
#include "div_by.h"
#include "pos_plan.h"

#include <type_traits>

#include <utility>

namespace bcnn {

struct MfmaArgs {
    ConvShape s;
    int32_t n_ptiles, n_ctiles;
    int32_t units_per_tap;  // cw / 4
    int32_t n_units;        // taps * cw / 4: 16-byte units along K that hold real data
    int32_t n_chunks;       // ceil(n_units / 2)
    int32_t z;              // 256 * n_chunks - K: positions that count +1 on their own
    int32_t x_bytes, w_bytes;  // sizes of the packed tensors, for the buffer descriptors
    int32_t row_jump;       // words added to the input offset when a filter row is complete
    int32_t tap_step;       // words added when a tap (branch) is complete: 0 for the plain convolution
    int32_t taps;           // filter taps = branches
    int32_t chunks_per_tap; // branch mode: cw / 8
    DivBy div_hw, div_wo;   // division of a pixel index by ho*wo and by wo
    DivBy div_ct;           // division of a tile index by n_ctiles
    PosArgs pos;            // position-major kernel only
};

// Branch mode (see the section in front of the fold below): per-branch scales,
// bias, what a tap outside the image stands for.
struct BranchEp {
    const float* scale;         // [taps][c_out]
    const float* bias;          // [c_out] or nullptr
    const uint32_t* pad_words;  // [taps][cw] (pad_mode 1)
    int32_t pad_mode;           // 0: -1 everywhere, 1: pad_words, 2: the tap contributes nothing
};
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
typedef int v2i __attribute__((ext_vector_type(2)));
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

// The loader's work of one chunk (the global -> LDS loads of the chunk fetched
// ahead and the bookkeeping around them) is cut into small statements, each
// issued behind a chosen MFMA of the chunk's slot program.  A wave issues in
// order and roughly one instruction per four cycles, so a 32-cycle MFMA hides
// about seven other instructions; bunched behind the first MFMAs of a chunk the
// loader left the matrix core idle.
//   K-steps 0-1: the loads.  Statement 0 is the weight block; then per input
//                block: validity mask / offset / load.  In order, each goes to
//                the next slot whose own fragment work leaves room (a slot
//                without a share of the weight expansion takes anything); all
//                are issued before the last slot of K-step 1, where the wave
//                waits for the chunk fetched earlier.
//   K-step 2   : the advance to the next fetch position, in four or five parts.
//   K-step 3   : the position of the next chunk's fetch (two parts) and the
//                bit counts of the weight words read ahead (two halves each).
template <int N> struct LoaderSlots { int v[N]; };
// instructions a slot holds anyway: two for its input half-fragment, three more where one of the
// eight weight-fragment registers of the next K-step falls into it
template <int NS> constexpr int slot_base(int slot)
{
    const int sl = slot % NS;
    return 2 + 3 * ((sl + 1) * 8 / NS - sl * 8 / NS);
}
template <int NS, int NWL, int NXL>     // NWL weight blocks and NXL input blocks per wave and chunk
constexpr LoaderSlots<NWL + 3 * NXL> loader_slots()
{
    constexpr int N = NWL + 3 * NXL;
    constexpr int CAP = 7;
    int cost[N] = {};
    for (int p = 0; p < NWL; ++p) cost[p] = 5;
    for (int p = 0; p < NXL; ++p) { cost[NWL + 3 * p] = 3; cost[NWL + 1 + 3 * p] = 1; cost[NWL + 2 + 3 * p] = 4; }
    int minbase = slot_base<NS>(0);
    for (int i = 1; i < NS; ++i) minbase = slot_base<NS>(i) < minbase ? slot_base<NS>(i) : minbase;
    const int last = 2 * NS - 2;
    LoaderSlots<N> r{};
    // (the chunk's first slots also carry what the loop's back edge leaves behind: start behind them)
    int slot = 2, used = slot_base<NS>(2);
    for (int j = 0; j < N; ++j) {
        while (!(used + cost[j] <= CAP || (used == slot_base<NS>(slot) && slot_base<NS>(slot) == minbase)) &&
               (last - slot) > (N - 1 - j)) {
            ++slot;
            used = slot_base<NS>(slot);
        }
        r.v[j] = slot;
        used += cost[j];
    }
    return r;
}
// n-th (from 1, up to 6) slot of a K-step that has no share of the weight expansion; evenly spread
// if there are fewer than six of those.  Increasing in n: statements placed by it keep their order.
template <int NS> constexpr int light_slot(int n)
{
    int light = 0;
    for (int sl = 0; sl < NS; ++sl) light += slot_base<NS>(sl) == 2;
    if (light < 6) return (n - 1) * NS / 6;
    int seen = 0;
    for (int sl = 0; sl < NS; ++sl)
        if (slot_base<NS>(sl) == 2 && ++seen == n) return sl;
    return NS - 1;
}

constexpr int PAD_LDS_WORDS = 9 * 64;   // pad words kept in LDS: taps * cw <= this
constexpr int MAX_BRANCHES = 16;        // scales kept in LDS: taps <= this

// PB = pixel blocks (of 32) per wave; the workgroup covers 2*32*PB pixels.
// Branch mode: OUT = OUT_BRANCH + 4 * pad mode + kind.  Pad mode: what a tap
// outside the image stands for (0: -1 everywhere, nothing to do; 1: the
// branch's pad words; 2: nothing at all).  Kind: what happens to the branch sum
// (float out, sign bits, or the module tail with a float / half real stream).
enum { OUT_I32 = 0, OUT_BITS = 1, OUT_MODULE_F32 = 2, OUT_MODULE_F16 = 3, OUT_MODULE_BF16 = 4, OUT_BRANCH = 8 };
enum { KIND_F32 = 0, KIND_BITS = 1, KIND_TAIL_F32 = 2, KIND_TAIL_F16 = 3 };

// PLAIN (module outputs outside branch mode only): the launcher has checked that
// every tile is whole along the channels, rows are vector aligned and identity,
// real stream and next bits are all present; the kernel then carries only the
// predicate-free epilogue (rows past the end are the one thing it still checks)
// instead of that and the general one: a third of the code, which a short
// kernel would otherwise spend its time fetching.
//
// POS: the tile is a run of pixel blocks of one segment of the position-major
// order (`pt`; a block = one output position in 32 consecutive images) and only
// the filter taps of the segment's rectangle are walked; see
// conv_mfma_fp4_pos_kernel.  `stage` is the workgroup's staging area in LDS,
// stage_units(PB) 16-byte units.
// NW = waves of the workgroup: 4 (2 along the channels x 2 along the pixels, the
// tile described above) or 2 (2 x 1: half the pixels, for tiles of finer grain;
// two such workgroups share a CU).
constexpr int stage_units(int pb, int nw = 4) { return 3 * (4 + (nw / 2) * pb) * 64; }

template <int PB, int OUT, bool EVEN, bool PLAIN, bool POS, int NW = 4>
__device__ __forceinline__ void conv_mfma_fp4_tile(
    const MfmaArgs& a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out, const ModuleEp& ep, const BranchEp& bp,
    uint4* stage, const int ptile, const int ctile, const PosTile& pt)
{
    static_assert(!POS || (OUT == OUT_BITS && EVEN && !PLAIN), "position-major tiles: fused output, whole chunks per tap");
    static_assert(NW == 4 || (NW == 2 && OUT == OUT_BITS), "two-wave workgroups: fused output only");
    constexpr int WP = NW / 2;        // waves along the pixels
    constexpr int NT = 64 * NW;       // threads
    constexpr bool FUSED = OUT == OUT_BITS;
    constexpr bool BRANCH = OUT >= OUT_BRANCH;
    constexpr int KIND = BRANCH ? (OUT - OUT_BRANCH) % 4 : -1;
    constexpr bool BRANCH_BITS = KIND == KIND_BITS;
    constexpr int PADMODE = BRANCH ? (OUT - OUT_BRANCH) / 4 : 0;       // 0: -1, 1: pad words, 2: skip
    static_assert(!BRANCH || EVEN, "branch mode needs whole chunks per tap");
    constexpr int WG_PX = 32 * WP * PB;
    // One stage = the chunk's 8 K-words of every row of the tile, as 16-byte
    // units (4 words = one K-half of a row).  Unit order: [block of 32 rows]
    // [K-half][row], blocks 0..3 weights, 4.. inputs; one wave-wide load fills
    // one block (1 KB), and lane l of a reader wave finds the words of its MFMA
    // row at unit 64*block + l.  Three stages rotate.
    constexpr int NBLK = 4 + WP * PB;            // blocks per stage
    constexpr int STAGE_BYTES = NBLK * 1024;
    constexpr int NWL = 4 / NW;                  // weight blocks a wave loads per chunk
    constexpr int NXL = (WP * PB + NW - 1) / NW; // input blocks
    constexpr int NL = NWL + NXL;                // loads per wave and chunk
    static_assert(3 * NBLK * 64 == stage_units(PB, NW), "size of the staging area");
    __shared__ __align__(16) float sub_lds[WG_CH];              // per channel: what the epilogue subtracts
    __shared__ int thr_lds[FUSED ? WG_CH : 1];                  // thresholds of the tile, fetched at kernel start
    // per tap: [parity][what the accumulator carries besides the tap's sum | the tap's sum where the tap is padding][channel]
    __shared__ __align__(16) float tapf_lds[BRANCH ? 2 : 1][2][WG_CH];
    __shared__ uint32_t pad_lds[BRANCH ? PAD_LDS_WORDS + 8 : 1];
    __shared__ __align__(16) float scale_lds[BRANCH ? MAX_BRANCHES : 1][WG_CH];   // scale[tap][channel of the tile]
    const ConvShape& s = a.s;
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wc = wave & 1, wp = wave >> 1;
    const int hsel = lane >> 5;
    const int j = lane & 31;

    const int o0 = ctile * WG_CH;
    const int m0 = ptile * WG_PX;   // (unused by position-major tiles)

    // The tile's thresholds are fetched now and parked in LDS behind the first
    // chunk's loads; the epilogue reads them there instead of waiting for global
    // memory after the last MFMA.
    int thr_early = 0;
    if constexpr (FUSED) {
        if (t < WG_CH) {
            const int ch = o0 + t;
            thr_early = thr[ch < s.c_out ? ch : s.c_out - 1];
        }
    }

    __shared__ int skip_lds[POS ? WG_CH : 1];   // position-major tiles: see below, behind the first loads
    if constexpr (POS) {
        if (t < WG_CH) skip_lds[t] = 0;
    }

    // ---- loader state.  Global -> LDS directly (buffer_load ... lds: lane l
    // of a wave writes 16 bytes at the LDS base of the instruction + 16*l, no
    // registers in between).  Per chunk wave w loads block w (weights) and the
    // input blocks w, w+4, ... ; lane l covers row l%32 of the block and the
    // K-half l/32 (even or odd 16-byte unit of the chunk).  A block index past
    // the end is clamped: the same data lands twice, which is harmless, and
    // every wave issues the same number of loads.
    int wrow_bytes[NWL];
#pragma unroll
    for (int i = 0; i < NWL; ++i) {
        int ch = o0 + 32 * (wave + NW * i) + row_to_channel(j);
        ch = ch < s.c_out ? ch : s.c_out - 1;
        wrow_bytes[i] = ch * a.n_units * 16;
    }
    // For input block i of this wave: word offset of the row's window top-left
    // tap (may point outside the image; only used where the tap's validity
    // bit is set) and one validity bit per tap.
    // One validity bit per tap (bit u*ks + v) of the window whose top-left input
    // position is (ph, pw).  The filter is 1x1 (no padding, every branch is
    // inside) or 3x3: three column bits, placed once per valid row.
    auto tap_mask = [&](int ph, int pw) -> uint32_t {
        if (s.ks == 1) return 0xFFFFFFFFu;
        uint32_t cols = 0, vm = 0;
#pragma unroll
        for (int v = 0; v < 3; ++v) cols |= (uint32_t)((uint32_t)(pw + v) < (uint32_t)s.w) << v;
#pragma unroll
        for (int u = 0; u < 3; ++u) vm |= ((uint32_t)(ph + u) < (uint32_t)s.h) ? cols << (3 * u) : 0u;
        return vm;
    };
    // Position-major tiles: block `bl` of the tile -> first image, output position; false past the
    // segment's end (the last block's numbers are returned then).  Wave-uniform when `bl` is.
    auto block_pos = [&](int bl, int& n0, int& oh, int& ow) -> bool { return pos_block(a.pos, pt, bl, n0, oh, ow); };
    int rbase[NXL];
    uint32_t vmask[NXL];
    int bblk[NXL];
#pragma unroll
    for (int i = 0; i < NXL; ++i) {
        int b = wave + NW * i;
        b = b < WP * PB ? b : WP * PB - 1;
        bblk[i] = b;
        const int row = 32 * b + j;
        int m = m0 + row;
        m = m < s.m ? m : s.m - 1;
        if constexpr (POS) {
            int n0, oh, ow;
            const bool active = block_pos(b, n0, oh, ow);
            const int ph = oh * s.stride - s.pad;
            const int pw = ow * s.stride - s.pad;
            rbase[i] = (((n0 + j) * s.h + ph) * s.w + pw) * s.cw;
            vmask[i] = active ? tap_mask(ph, pw) : 0u;     // a block past the end fetches nothing
        } else if (s.ks == 1 && s.stride == 1) {   // 1x1, unit stride: output pixel m is input pixel m, no divisions
            rbase[i] = m * s.cw;
            vmask[i] = 0xFFFFFFFFu;
        } else {
            const int hw = s.ho * s.wo;
            const int n = a.div_hw(m);
            const int r = m - n * hw;
            const int oh = a.div_wo(r);
            const int ph = oh * s.stride - s.pad;
            const int pw = (r - oh * s.wo) * s.stride - s.pad;
            rbase[i] = ((n * s.h + ph) * s.w + pw) * s.cw;
            vmask[i] = tap_mask(ph, pw);
        }
    }

    // ---- position of the chunk to fetch next along K.
    // Lanes 0-31 fetch the chunk's even 16-byte unit, lanes 32-63 the odd one.
    // All of it is wave-uniform scalar arithmetic without selects or division
    // (compare results used as 0/1 factors), so it never branches and costs
    // the vector ALU nothing.
    //   EVEN (units per tap even: C_in a multiple of 256): both units of a
    //     chunk lie in one tap, 16 bytes apart, so one (tap, offset) pair
    //     serves the wave and the lanes' halves are folded into rbase/wrow.
    //     Past the last chunk the position stops advancing: the extra fetches
    //     of the pipeline's tail reload the last chunk's inputs (and zeros for
    //     the weights) into stages whose contents are never multiplied.
    //   otherwise: the two units are tracked separately and each lane selects
    //     its own; units past the end (K padding) read as zero.
    //   position-major tiles walk the taps (u, v) of the rectangle u_lo .. u_lo+nu-1 x v_lo .. v_lo+nv-1
    //     only: `tap` stays the tap's number in the full filter (the validity bits are indexed by
    //     it), the weights' offset `woff` is tracked beside the inputs' and both jump at the end of
    //     a filter row.
    const int row_jump = POS ? (s.w - pt.nv) * s.cw : a.row_jump;
    const int w_row_jump = POS ? (s.ks - pt.nv) * s.cw * 4 : 0;     // bytes
    const int n_chunks = POS ? pt.nu * pt.nv * (a.units_per_tap >> 1) : a.n_chunks;
    const int taps_per_row = POS ? pt.nv : s.ks;
    struct KPos { int unit, tap, v, ut, off, woff; };
    KPos k0 = {0, 0, 0, 0, 0, 0}, k1 = {0, 0, 0, 0, 0, 0};
    if constexpr (POS) {
        k0.tap = pt.u_lo * s.ks + pt.v_lo;
        k0.off = (pt.u_lo * s.w + pt.v_lo) * s.cw;
        k0.woff = k0.tap * s.cw * 4;
    }
    auto advance1 = [&](KPos& p, int per_tap, int step_words, int go) {
        const int ut1 = p.ut + go;
        const int tap_done = ut1 == per_tap ? 1 : 0;
        p.ut = ut1 * (1 - tap_done);
        p.tap += tap_done;
        const int v1 = p.v + tap_done;
        const int row_done = v1 == s.ks ? 1 : 0;
        p.v = v1 * (1 - row_done);
        p.off += go * step_words + row_done * row_jump + tap_done * a.tap_step;
        p.unit += go;
    };
    if constexpr (!EVEN) advance1(k1, a.units_per_tap, 4, 1);
    int fetched = 0;   // chunks fetched so far (EVEN only)
    auto advance = [&]() {
        if constexpr (POS) {
            fetched += 1;
            const int go = k0.unit + 1 < n_chunks ? 1 : 0;
            const int ut1 = k0.ut + go;
            const int tap_done = ut1 == (a.units_per_tap >> 1) ? 1 : 0;
            k0.ut = ut1 * (1 - tap_done);
            const int v1 = k0.v + tap_done;
            const int row_done = v1 == taps_per_row ? 1 : 0;
            k0.v = v1 * (1 - row_done);
            k0.tap += tap_done + row_done * (s.ks - taps_per_row);
            k0.off += go * 8 + row_done * row_jump;
            k0.woff += go * 32 + row_done * w_row_jump;
            k0.unit += go;
        } else if constexpr (EVEN) {
            fetched += 1;
            // k0.unit counts chunks here; stop on the last one
            advance1(k0, a.units_per_tap >> 1, 8, k0.unit + 1 < n_chunks ? 1 : 0);
        } else {
            advance1(k0, a.units_per_tap, 4, 1); advance1(k0, a.units_per_tap, 4, 1);
            advance1(k1, a.units_per_tap, 4, 1); advance1(k1, a.units_per_tap, 4, 1);
        }
    };
    if constexpr (EVEN) {   // fold the lane's K-half into its base offsets
#pragma unroll
        for (int i = 0; i < NWL; ++i) wrow_bytes[i] += 16 * hsel;
#pragma unroll
        for (int i = 0; i < NXL; ++i) rbase[i] += 4 * hsel;
    }

    // ---- global -> LDS loads.
    // A lane whose unit must read as zero (out-of-image tap, K padding past
    // the last real unit) gets the offset -16, beyond any buffer: the hardware
    // range check makes the load deliver 0, so the loader has no branches.
    // The loads are written as inline assembly on purpose: the compiler's
    // wait-count pass treats every later LDS read as possibly aliasing a
    // pending global->LDS load and would force vmcnt(0) in front of it, which
    // serialises the pipeline.  Written this way the compiler does not see
    // them, and the explicit s_waitcnt vmcnt(N) before each barrier below is
    // what orders them (N = loads that may still be in flight).  M0 carries
    // the LDS destination; nothing else in this kernel uses M0.  The v_bfi
    // between the M0 write and the load (offset = mask ? offset : -16) also
    // fills the wait state that pair needs.
    auto make_rsrc = [](const void* base, int bytes) -> v4i {
        const uint64_t p = reinterpret_cast<uint64_t>(base);
        // dword 1: address bits 47:32, stride 0; dword 3: 32-bit untyped data format
        return v4i{(int)(uint32_t)p, (int)((uint32_t)(p >> 32) & 0xFFFFu), bytes, 0x00020000};
    };
    const v4i xres = make_rsrc(x, a.x_bytes);
    const v4i wres = make_rsrc(w, a.w_bytes);
    const uint32_t stage_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)stage;
    // LDS byte addresses, within a stage, of the blocks this wave fills (`buf` below is a stage's byte offset)
    uint32_t w_lds[NWL];
#pragma unroll
    for (int i = 0; i < NWL; ++i) w_lds[i] = stage_lds + (uint32_t)(wave + NW * i) * 1024u;
    uint32_t x_lds[NXL];
#pragma unroll
    for (int i = 0; i < NXL; ++i) x_lds[i] = stage_lds + (uint32_t)(4 + bblk[i]) * 1024u;
    auto dma16 = [&](const v4i& rsrc, uint32_t lds_byte, uint32_t offset, uint32_t mask) {
        uint32_t tmp;
        // wave-uniform by construction; the compiler may still park it in a vector register when
        // scalar registers run short, and the "s" constraint alone does not move it back
        const uint32_t lds_s = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_byte);
        asm volatile("s_mov_b32 m0, %1\n\tv_bfi_b32 %0, %3, %2, -16\n\tbuffer_load_dwordx4 %0, %4, 0 offen lds"
                     : "=&v"(tmp) : "s"(lds_s), "v"(offset), "v"(mask), "s"(rsrc) : "memory");
    };
    // per chunk, before its fetch_piece calls
    int f_real = -1, f_tap = 0, f_off = 0, f_woff = 0;
    auto fetch_begin = [&]() {
        if constexpr (EVEN) {
            // weights of a chunk past the end must read as zero: the readers
            // count the set bits of every weight word that passes through
            f_real = -(fetched < n_chunks ? 1 : 0);
            f_tap = k0.tap;
            f_off = k0.off;
            f_woff = POS ? k0.woff : k0.unit * 32;
        } else {
            const int unit = hsel ? k1.unit : k0.unit;
            f_real = unit < a.n_units ? -1 : 0;
            f_tap = hsel ? k1.tap : k0.tap;
            f_off = hsel ? k1.off : k0.off;
            f_woff = unit * 16;
        }
    };
    // f_woff: byte offset along K of the chunk within a weight row
    auto fetch_piece = [&](int buf, int i) {  // i < NWL: weight blocks; then the input blocks
        if (i < NWL) {
            dma16(wres, w_lds[i] + (uint32_t)buf, (uint32_t)(wrow_bytes[i] + f_woff), (uint32_t)f_real);
        } else {
            // validity bit of the tap, sign-extended to a mask
            int m = __builtin_amdgcn_sbfe((int)vmask[i - NWL], (uint32_t)f_tap & 31u, 1u);
            m &= f_real;     // chunks past the end fetch nothing (an out-of-range offset returns 0 at once)
            dma16(xres, x_lds[i - NWL] + (uint32_t)buf,
                  (uint32_t)(rbase[i - NWL] + f_off) << 2, (uint32_t)m);
        }
    };

    // The same work cut into statements for the chunk loop (see loader_slots()).
    constexpr int ADV_STMTS = EVEN ? 5 : 4;
    constexpr int N_PIECE = NWL + 3 * NXL;
    int p_mask = 0;
    uint32_t p_off = 0;
    int adv_go = 0, adv_td = 0, adv_rd = 0;
    auto piece_stmt = [&](auto jc, int buf) {
        constexpr int j = decltype(jc)::value;
        if constexpr (j < NWL) {
            fetch_piece(buf, j);
        } else {
            constexpr int pi = (j - NWL) / 3, part = (j - NWL) % 3;      // input block pi of this wave
            if constexpr (part == 0) {
                p_mask = __builtin_amdgcn_sbfe((int)vmask[pi], (uint32_t)f_tap & 31u, 1u) & f_real;
            } else if constexpr (part == 1) {
                p_off = (uint32_t)(rbase[pi] + f_off) << 2;
            } else {
                dma16(xres, x_lds[pi] + (uint32_t)buf, p_off, (uint32_t)p_mask);
            }
        }
    };
    auto advance_stmt = [&](auto kc) {
        constexpr int part = decltype(kc)::value;
        if constexpr (EVEN) {            // advance() in five parts
            if constexpr (part == 0) {
                adv_go = k0.unit + 1 < n_chunks ? 1 : 0;   // k0.unit counts chunks here; stop on the last one
            } else if constexpr (part == 1) {
                const int ut1 = k0.ut + adv_go;
                adv_td = ut1 == (a.units_per_tap >> 1) ? 1 : 0;
                k0.ut = adv_td ? 0 : ut1;
            } else if constexpr (part == 2) {
                const int v1 = k0.v + adv_td;
                adv_rd = v1 == taps_per_row ? 1 : 0;
                k0.v = adv_rd ? 0 : v1;
                k0.tap += adv_td;
                if constexpr (POS) k0.tap += adv_rd ? s.ks - taps_per_row : 0;
            } else if constexpr (part == 3) {
                k0.off += (adv_go ? 8 : 0) + (POS ? 0 : (adv_td ? a.tap_step : 0));
                if constexpr (POS) k0.woff += adv_go ? 32 : 0;
            } else {
                k0.off += adv_rd ? row_jump : 0;
                if constexpr (POS) k0.woff += adv_rd ? w_row_jump : 0;
                k0.unit += adv_go;
                fetched += 1;
            }
        } else {
            advance1(part < 2 ? k0 : k1, a.units_per_tap, 4, 1);
        }
    };
    auto begin_stmt = [&](auto kc) {     // fetch_begin() in two parts
        constexpr int part = decltype(kc)::value;
        if constexpr (part == 0) {
            if constexpr (EVEN) {
                f_real = -(fetched < n_chunks ? 1 : 0);
                f_tap = k0.tap;
                f_off = k0.off;
            } else {
                const int unit = hsel ? k1.unit : k0.unit;
                f_real = unit < a.n_units ? -1 : 0;
                f_tap = hsel ? k1.tap : k0.tap;
                f_off = hsel ? k1.off : k0.off;
            }
        } else {
            if constexpr (POS) f_woff = k0.woff;
            else if constexpr (EVEN) f_woff = k0.unit * 32;
            else f_woff = (hsel ? k1.unit : k0.unit) * 16;
        }
    };

    // ---- branch mode: F x F as F*F shifted binary 1x1 branches (or P parallel
    // 1x1 branches), each with its own real scale per output channel (BCNN
    // paper, Section 4.2.1, last paragraph; Figure 2, bottom).  A tap's chunks
    // accumulate in `acc` as usual; when the tap is complete its exact integer
    // sum y_t = acc - (2*pop_t(channel) - 192*chunks_per_tap) is folded into the
    // float totals, tot = fma(scale[t][channel], y_t, tot), and acc restarts at
    // zero.  pop_t are the weight-bit counts of that tap alone, exchanged
    // through LDS at every fold.  A pixel whose tap lies outside the image has
    // read all-zero words (-1 everywhere); where the tap should stand for the
    // branch's pad words instead, its y_t is replaced by c_in - 2*popcount(pad
    // words xor weights), which the weight readers count on the way like pop_t;
    // where it should contribute nothing the fold is skipped for that pixel.
    v16f tot[BRANCH ? CB : 1][BRANCH ? PB : 1];
    uint32_t vmask_d[PB];
    auto branch_channel = [&](int cb, int r) {
        const int ch = o0 + 64 * wc + 32 * cb + 16 * hsel + r;
        return ch < s.c_out ? ch : s.c_out - 1;
    };
    if constexpr (BRANCH) {
        for (int i = t; i < a.taps * WG_CH; i += NT) {
            const int tp = i / WG_CH, cl = i - tp * WG_CH;
            const int ch = o0 + cl < s.c_out ? o0 + cl : s.c_out - 1;
            scale_lds[tp][cl] = bp.scale[(size_t)tp * s.c_out + ch];
        }
        for (int i = t; i < PAD_LDS_WORDS + 8; i += NT)
            pad_lds[i] = (PADMODE == 1 && i < a.taps * s.cw) ? bp.pad_words[i] : 0u;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float b = bp.bias ? bp.bias[branch_channel(cb, r)] : 0.0f;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) tot[cb][pb][r] = b;
            }
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            int m = m0 + 32 * (PB * wp + pb) + j;
            m = m < s.m ? m : s.m - 1;
            const int hw = s.ho * s.wo;
            const int r = m - a.div_hw(m) * hw;
            const int oh = a.div_wo(r);
            const int ph = oh * s.stride - s.pad;
            const int pw_ = (r - oh * s.wo) * s.stride - s.pad;
            vmask_d[pb] = tap_mask(ph, pw_);
        }
    }

    // ---- accumulators: lane (pixel j = lane%32, half h = lane/32), register r
    //      <-> channel 32*block + 16h + r.  They start at zero; every constant
    //      and per-channel term is applied in the epilogue.
    //      (They are cleared further down, between the issue of the first loads
    //      and the wait for them.)
    v16f acc[CB][PB];

    // ---- module output: is this workgroup's tile the plain case (whole tile
    // inside the output, vector-aligned rows, identity / real stream / next bits
    // all present)?  Then its epilogue runs without per-element predicates, and
    // the identity vectors of the first pixel block(s) are fetched right here,
    // so that their trip to HBM hides behind the K loop instead of starting
    // after it (the real stream may be updated in place: these are reads of
    // elements only this workgroup writes, and it writes them later).
    constexpr bool MODULE = (OUT >= OUT_MODULE_F32 && OUT <= OUT_MODULE_BF16) || KIND >= KIND_TAIL_F32;
    // storage type of the real stream (branch mode: float or half)
    constexpr int REAL = OUT == OUT_MODULE_BF16 ? REAL_BF16 : (OUT == OUT_MODULE_F16 || KIND == KIND_TAIL_F16) ? REAL_F16 : REAL_F32;
    constexpr bool HALF = REAL != REAL_F32;                // a 16-bit stream
    // (only where 32 registers can be held through the loop: the half-precision stream outside branch mode)
    constexpr bool EARLY_IDS = MODULE && !BRANCH && HALF;
    using real_t = typename real_type<REAL>::type;
    typedef real_t real4 __attribute__((ext_vector_type(4)));
    constexpr int AHEAD = HALF ? 2 : 1;                    // pixel blocks in flight ahead of the one in work
    real4 early_ids[EARLY_IDS ? AHEAD : 1][8];
    static_assert(!PLAIN || (MODULE && !BRANCH), "PLAIN is a module-output variant");
    // The plain case addresses the identity, the real stream and the next bits as raw buffers, one
    // descriptor per wave and tensor: base = the row of the wave's first pixel, size = the wave's rows
    // that exist.  A lane's byte offset is then a 32-bit constant plus the row's (wave-uniform) offset,
    // a row past the end of the tensor reads zeros and stores nothing, and a lane that has nothing to
    // store uses an offset past every size: no 64-bit address arithmetic and no predicates per row.
    auto wave_rows_rsrc = [&](const void* base, int row_bytes) {
        const int m_w = m0 + 32 * PB * wp;
        int rows = s.m - m_w;
        rows = rows < 0 ? 0 : (rows > 32 * PB ? 32 * PB : rows);
        const uint64_t at = reinterpret_cast<uint64_t>(base) + (uint64_t)m_w * (uint64_t)row_bytes;
        // wave-uniform by construction; said explicitly so that the descriptor is built in scalar registers
        const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)at);
        const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(at >> 32));
        return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<char*>((hi << 32) | lo), 0,
                                                 __builtin_amdgcn_readfirstlane(rows * row_bytes), 0x00020000);
    };
    auto load_real4 = [](__amdgpu_buffer_rsrc_t res, uint32_t lane_off, int row_off) -> real4 {
        if constexpr (HALF)      // aux 2: streamed once, non-temporal
            return __builtin_bit_cast(real4, __builtin_amdgcn_raw_buffer_load_b64(res, (int)(lane_off + (uint32_t)row_off), 0, 2));
        else
            return __builtin_bit_cast(real4, __builtin_amdgcn_raw_buffer_load_b128(res, (int)(lane_off + (uint32_t)row_off), 0, 2));
    };
    bool module_fast = PLAIN;
    if constexpr (MODULE) {
        if constexpr (BRANCH) {      // branch mode decides per workgroup and carries both epilogues
            const uintptr_t both = reinterpret_cast<uintptr_t>(ep.r) | reinterpret_cast<uintptr_t>(ep.identity);
            module_fast = ep.identity && ep.r && ep.x_next && s.c_out % 4 == 0 && ep.id_channels % 4 == 0 &&
                          s.c_out <= (1 << 20) &&
                          (both & (HALF ? 7 : 15)) == 0 && m0 + WG_PX <= s.m && o0 + WG_CH <= s.c_out;
        }
        if constexpr (EARLY_IDS) {
            if (module_fast) {
                const int e_c0 = o0 + 64 * wc + 4 * (lane & 15);
                const uint32_t e_voff = (uint32_t)(((lane >> 4) * ep.id_channels + e_c0 % ep.id_channels) *
                                                   (int)sizeof(real_t));
                const auto e_res = wave_rows_rsrc(ep.identity, ep.id_channels * (int)sizeof(real_t));
#pragma unroll
                for (int k = 0; k < AHEAD && k < PB; ++k)
#pragma unroll
                    for (int g = 0; g < 8; ++g)
                        early_ids[k][g] = load_real4(e_res, e_voff, (32 * k + 4 * g) * ep.id_channels * (int)sizeof(real_t));
            }
        }
    }

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
    //   K-steps 0-1: global -> LDS loads of chunk c+2, a few instructions per
    //                slot (loader_slots())
    //   K-step 1   : at its end, wait for this wave's loads of chunk c+1
    //                (issued at least four K-steps earlier) and workgroup barrier
    //   K-step 2   : LDS reads of chunk c+1's weight words; the loader advances
    //   K-step 3   : LDS reads of chunk c+1's input words, each block's right
    //                after that block's last use; position of chunk c+3's fetch
    // Stage c%3 holds chunk c.  All of it is read during chunk c-1, whose
    // end every wave has reached behind chunk c's barrier; chunk c+3's loads
    // are issued a whole chunk after that.
    constexpr int NF = CB + PB;       // words per lane and K-step: weights first, then inputs
    constexpr int NS = CB * PB;       // MFMA slots per K-step
    constexpr auto LSLOTS = loader_slots<NS, NWL, NXL>();
    static_assert(LSLOTS.v[N_PIECE - 1] <= 2 * NS - 2, "the loads must be issued before the wait of K-step 1");
    static_assert(light_slot<NS>(ADV_STMTS + 1) < NS && light_slot<NS>(2 + 2 * CB) < NS, "bookkeeping slots must exist");
    static_assert(light_slot<NS>(1) < light_slot<NS>(2) && light_slot<NS>(2) < light_slot<NS>(3) &&
                  light_slot<NS>(3) < light_slot<NS>(4) && light_slot<NS>(4) < light_slot<NS>(5) &&
                  light_slot<NS>(5) < light_slot<NS>(6), "bookkeeping statements must keep their order");
    static_assert(CB == 2, "slot program assumes two channel blocks");
    // the fragments of the next chunk's blocks 0 and 1 are expanded behind pixel blocks PB-2 and PB-1 of
    // K-step 3, from words re-read behind blocks 0 and 1 of the same K-step: that needs a few slots between
    static_assert(PB >= 4, "slot program needs at least four pixel blocks per wave");
    static_assert(NL + 2 <= NS && NF <= NS && 2 * NL <= 15, "side work must fit the MFMA slots of a K-step");
    const Fp4Masks masks = fp4_masks();
    int fa[2][CB][4];                 // weight fragments, double buffered over K-steps
    int fb[4][4];                     // input fragments, ring over (K-step, pixel block)
    uint4 pw[NF];                     // this lane's four words (K-steps 0..3) of the chunk, per block
    uint4 pwn[CB];                    // the next chunk's weight words (read before the current ones retire)
    int wpop[CB] = {0, 0};            // set weight bits at positions 4i+0..2 of this lane's rows
    const char* lds0 = reinterpret_cast<const char*>(stage) + lane * 16;
    // One ds_read_b128 per block and chunk: lanes read consecutive 16-byte
    // units, which is conflict free.  The next chunk's words replace a block's
    // words during K-step 3, right after their last use.
    auto read_unit = [&](uint4& dst, int buf, int f) {
        const int blk = f < CB ? 2 * wc + f : 4 + PB * wp + (f - CB);
        dst = *reinterpret_cast<const uint4*>(lds0 + buf + blk * 1024);
    };
    // Branch mode keeps the counts of the chunk read ahead apart (wnext, wpadn)
    // until the chunk loop knows which tap they belong to; wpadn counts the
    // positions where the weights differ from the tap's pad words (padq: this
    // lane's four pad words of that chunk).
    int wnext[CB] = {0, 0}, wpad[CB] = {0, 0}, wpadn[CB] = {0, 0};
    uint4 padq = make_uint4(0u, 0u, 0u, 0u);
    int cnt_half[CB] = {0, 0};
    auto count_unit_half = [&](const uint4& q, int f, int half) {   // the same in two halves for the chunk loop
        if (half == 0) {
            cnt_half[f] = __builtin_popcount(q.x & 0x77777777u) + __builtin_popcount(q.y & 0x77777777u);
            return;
        }
        const int c = cnt_half[f] + __builtin_popcount(q.z & 0x77777777u) + __builtin_popcount(q.w & 0x77777777u);
        if constexpr (BRANCH) {
            wnext[f] = c;
            if constexpr (PADMODE == 1)
                wpadn[f] = __builtin_popcount(q.x ^ padq.x) + __builtin_popcount(q.y ^ padq.y) +
                           __builtin_popcount(q.z ^ padq.z) + __builtin_popcount(q.w ^ padq.w);
        } else {
            wpop[f] += c;
        }
    };
    auto count_unit = [&](const uint4& q, int f) {   // well after the read, so nothing waits
        const int c = __builtin_popcount(q.x & 0x77777777u) + __builtin_popcount(q.y & 0x77777777u) +
                      __builtin_popcount(q.z & 0x77777777u) + __builtin_popcount(q.w & 0x77777777u);
        if constexpr (BRANCH) {
            wnext[f] = c;
            if constexpr (PADMODE == 1)
                wpadn[f] = __builtin_popcount(q.x ^ padq.x) + __builtin_popcount(q.y ^ padq.y) +
                           __builtin_popcount(q.z ^ padq.z) + __builtin_popcount(q.w ^ padq.w);
        } else {
            wpop[f] += c;
        }
    };
    auto word_of = [&](int f, int ks) -> uint32_t {   // ks = 0..3 within the chunk
        return ks == 0 ? pw[f].x : ks == 1 ? pw[f].y : ks == 2 ? pw[f].z : pw[f].w;
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
    // the same holds for the next chunk.  b1/b2 = stages of chunk c+1, c+2.
    auto chunk_body = [&](int b1, int b2) {
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
                if constexpr (ks < 3) fa[(ks + 1) & 1][f][jj] = expand_w(word_of(f, ks + 1), jj);
                else fa[0][f][jj] = expand_w(pwn[f].x, jj);
            });
            // side work, spread over the slots of its K-step
            if constexpr (ks == 1 && sl == NS - 1) {
                // outstanding: this wave's loads of chunks c+1 and c+2, NL each, in order
                asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NL) : "memory");   // chunk c+1 has landed
                __syncthreads();
            }
            // chunk c+1's words: weights early in K-step 2 (into the spare
            // set), input block pb in K-step 3 right after the block's last use
            if constexpr (ks == 2 && sl < CB) read_unit(pwn[sl], b1, sl);
            if constexpr (ks == 3 && cb == 1) read_unit(pw[CB + pb], b1, CB + pb);
            // chunk c+2's loads, then the loader's bookkeeping for chunk c+3, a statement at a time
            static_for<N_PIECE>([&](auto jc) {
                if constexpr (LSLOTS.v[decltype(jc)::value] == i) piece_stmt(jc, b2);
            });
            static_for<ADV_STMTS>([&](auto kc) {
                if constexpr (i == 2 * NS + light_slot<NS>(decltype(kc)::value + 2)) advance_stmt(kc);
            });
            static_for<2>([&](auto kc) {
                if constexpr (i == 3 * NS + light_slot<NS>(decltype(kc)::value + 1)) begin_stmt(kc);
            });
            static_for<2 * CB>([&](auto kc) {        // bit counts of the weight words read in K-step 2
                constexpr int k = decltype(kc)::value;
                if constexpr (i == 3 * NS + light_slot<NS>(k + 3)) count_unit_half(pwn[k >> 1], k >> 1, k & 1);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
#pragma unroll
        for (int f = 0; f < CB; ++f) pw[f] = pwn[f];
    };

#pragma unroll
    for (int c = 0; c < 2; ++c) {                        // chunks 0, 1 -> stages 0, 1
        fetch_begin();
#pragma unroll
        for (int i = 0; i < NL; ++i) fetch_piece(c * STAGE_BYTES, i);
        advance();
    }
    fetch_begin();                                       // chunk 2: the loop expects its position ready
    // Position-major tiles: what the taps that are not walked add to every pixel of the tile, per
    // channel.  Such a tap is outside the image for all of them, i.e. -1 in every channel: its sum is
    // c_in - 2 * popcount(the tap's weight words).  skip_lds[channel] collects the popcounts.  The
    // workgroup's threads run over (channel, 16-byte unit) of a tap, neighbouring lanes on
    // neighbouring units; a thread's place in that order does not depend on the tap, so its offsets
    // are computed once and the taps only add a wave-uniform term.  The loads of three taps (an edge
    // misses one filter row or column) are in flight together: one trip to memory, which at the
    // start of a kernel is some 4000 cycles.  They are issued behind the first chunks' loads so that
    // the two waits overlap: loads complete in order, so the wait for these also covers the
    // loader's, whose own wait (counted by hand) then finds nothing left.
    if constexpr (POS) {
        const int n_skip = s.ks * s.ks - pt.nu * pt.nv;
        if (n_skip > 0) {
            __syncthreads();                                        // skip_lds is cleared
            uint64_t list = 0;                                      // the skipped taps, four bits each
            {
                int cnt = 0;
                for (int u = 0; u < s.ks; ++u)
                    for (int v = 0; v < s.ks; ++v) {
                        const bool walked = u >= pt.u_lo && u < pt.u_lo + pt.nu && v >= pt.v_lo && v < pt.v_lo + pt.nv;
                        if (!walked) { list |= (uint64_t)(u * s.ks + v) << (4 * cnt); cnt += 1; }
                    }
            }
            const int per_tap = s.cw >> 2;                          // 16-byte units of a tap
            const int per_wg = WG_CH * per_tap;                     // of a tap over the tile's channels
            const int rounds = (per_wg + NT - 1) / NT;              // per thread and tap
            const auto wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(w), 0, a.w_bytes, 0x00020000);
            constexpr int RMAX = 1024 / NT, TU = 3;
            for (int r0 = 0; r0 < rounds; r0 += RMAX) {
                int off[RMAX], cl[RMAX], pop[RMAX];
#pragma unroll
                for (int k = 0; k < RMAX; ++k) {
                    const int e = t + (r0 + k) * NT;
                    const bool ok = r0 + k < rounds && e < per_wg;
                    cl[k] = a.pos.div_per_tap(ok ? e : 0);
                    const int q = (ok ? e : 0) - cl[k] * per_tap;
                    const int ch = o0 + cl[k] < s.c_out ? o0 + cl[k] : s.c_out - 1;
                    off[k] = ok ? (ch * (s.ks * s.ks) * per_tap + q) * 16 : -1;   // negative: reads nothing
                    pop[k] = 0;
                }
                for (int g0 = 0; g0 < n_skip; g0 += TU) {
                    v4i d[TU][RMAX];
#pragma unroll
                    for (int g = 0; g < TU; ++g) {
                        const int gi = g0 + g < n_skip ? g0 + g : n_skip - 1;
                        const int tap_off = (int)((list >> (4 * gi)) & 15u) * per_tap * 16;
                        const bool real = g0 + g < n_skip;
#pragma unroll
                        for (int k = 0; k < RMAX; ++k)   // offsets past the tensor read as zero: no bits
                            d[g][k] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(
                                wbuf, (real && off[k] >= 0) ? off[k] + tap_off : -16, 0, 0));
                    }
#pragma unroll
                    for (int g = 0; g < TU; ++g)
#pragma unroll
                        for (int k = 0; k < RMAX; ++k)
                            pop[k] += __builtin_popcount((uint32_t)d[g][k][0]) + __builtin_popcount((uint32_t)d[g][k][1]) +
                                      __builtin_popcount((uint32_t)d[g][k][2]) + __builtin_popcount((uint32_t)d[g][k][3]);
                }
#pragma unroll
                for (int k = 0; k < RMAX; ++k) atomicAdd(&skip_lds[cl[k]], pop[k]);
            }
        }
    }

    // The accumulators are cleared here, while the first chunks are on their way from memory.  Left to
    // itself the compiler re-creates the zeros right in front of the loop, after the wait; the empty
    // statements below take every accumulator as input and output, so the zeros must exist here.
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;
            // (branch mode holds a second accumulator set; pinning this one to a register class there
            // leaves the allocator no room and it spills, so the compiler places those zeros itself)
            if constexpr (BRANCH) continue;
            else if constexpr (PB >= 6) asm volatile("" : "+a"(acc[cb][pb]));     // the wide tiles keep them in acc registers
            else asm volatile("" : "+v"(acc[cb][pb]));
        }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (FUSED) {
        // |y| <= K, so thresholds beyond +-(K+1) decide nothing new and are clamped
        if (t < WG_CH)
            thr_lds[t] = thr_early > s.k + 1 ? s.k + 1 : (thr_early < -s.k - 1 ? -s.k - 1 : thr_early);
    }
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(NL) : "memory");   // chunk 0 has landed
    __syncthreads();
#pragma unroll
    for (int f = 0; f < NF; ++f) read_unit(pw[f], 0, f);
    if constexpr (PADMODE == 1) padq = *reinterpret_cast<const uint4*>(pad_lds + 4 * hsel);   // chunk 0
#pragma unroll
    for (int f = 0; f < CB; ++f) {
        count_unit(pw[f], f);
        if constexpr (BRANCH) { wpop[f] = wnext[f]; wpad[f] = wpadn[f]; }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) fa[0][f][jj] = expand_w(pw[f].x, jj);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) fb[q][jj] = expand_x(pw[CB + q].x, jj);

    {
        int b0 = 0, b1 = STAGE_BYTES, b2 = 2 * STAGE_BYTES;   // byte offsets of the three stages
        int tap = 0, chunk_in_tap = 0, par = 0;
        const int c_in = 256 * a.chunks_per_tap;
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            if constexpr (PADMODE == 1)   // pad words of the chunk whose weights this body reads ahead
                padq = *reinterpret_cast<const uint4*>(pad_lds + 8 * (chunk + 1) + 4 * hsel);
            chunk_body(b1, b2);
            const int tmp = b0; b0 = b1; b1 = b2; b2 = tmp;
            if constexpr (BRANCH) {
                chunk_in_tap += 1;
                if (chunk_in_tap < a.chunks_per_tap) {
#pragma unroll
                    for (int f = 0; f < CB; ++f) { wpop[f] += wnext[f]; wpad[f] += wpadn[f]; }
                    continue;
                }
                // ---- the tap is complete: fold it
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    // lanes l and l^32 read the two K-halves of the same weight row
                    const int both = wpop[cb] + __shfl_xor(wpop[cb], 32, 64);
                    const int bothp = wpad[cb] + __shfl_xor(wpad[cb], 32, 64);
                    if (hsel == 0) {          // one lane per channel turns the counts into the two terms
                        const int ch = 64 * wc + 32 * cb + row_to_channel(j);
                        tapf_lds[par][0][ch] = (float)(2 * both - 192 * a.chunks_per_tap);
                        if constexpr (PADMODE == 1) tapf_lds[par][1][ch] = (float)(c_in - 2 * bothp);
                    }
                    wpop[cb] = wnext[cb];
                    wpad[cb] = wpadn[cb];
                }
                __syncthreads();
                // the lane's 16 channels of a block are consecutive: four 16-byte reads per table
                typedef float f4v __attribute__((ext_vector_type(4)));
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int cl4 = 64 * wc + 32 * cb + 16 * hsel + (r & ~3);
                        const f4v corr4 = *reinterpret_cast<const f4v*>(&tapf_lds[par][0][cl4]);
                        const f4v g4 = *reinterpret_cast<const f4v*>(&scale_lds[tap][cl4]);
                        const float corr = corr4[r & 3];
                        const float g = g4[r & 3];
                        float ypad = 0.0f;
                        if constexpr (PADMODE == 1) {
                            const f4v ypad4 = *reinterpret_cast<const f4v*>(&tapf_lds[par][1][cl4]);
                            ypad = ypad4[r & 3];
                        }
#pragma unroll
                        for (int pb = 0; pb < PB; ++pb) {
                            const bool inb = PADMODE == 0 || ((vmask_d[pb] >> tap) & 1u);
                            float y = acc[cb][pb][r] - corr;
                            if constexpr (PADMODE == 1) y = inb ? y : ypad;
                            const float zn = __builtin_fmaf(g, y, tot[cb][pb][r]);
                            if constexpr (PADMODE == 2) tot[cb][pb][r] = inb ? zn : tot[cb][pb][r];
                            else tot[cb][pb][r] = zn;
                            acc[cb][pb][r] = 0.0f;
                        }
                        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // keep the live set small
                    }
                tap += 1;
                chunk_in_tap = 0;
                par ^= 1;
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // drain the loads of the chunks past the end

    // ---- epilogue
    // The accumulator holds  sum + Z - 192*n_chunks + 2*pop(channel)  (Z:
    // positions that are zero on both sides and count +1, see the launcher;
    // pop: the channel's set weight bits at positions 4i+0..2, see the
    // header).  The two lanes that read a weight row's K-halves add their
    // counts and the workgroup exchanges them through LDS indexed by channel.  What
    // has to be subtracted per channel (plus the threshold, minus 0.5 so that
    // the result is never zero, in the fused case) is kept in sub[][].
    float sub[CB][16];
    if constexpr (!BRANCH) {
        // The lane that holds a channel's count turns it into the value to subtract and leaves it in
        // LDS as a float; every lane then fetches its 2 x 16 channels with eight 16-byte reads.
        // (position-major tiles: Z counts the walked taps only)
        const int base = (POS ? pt.nu * pt.nv * a.pos.z_per_tap : a.z) - 192 * n_chunks;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            // lanes l and l^32 read the two K-halves of the same weight row
            const int both = wpop[cb] + __shfl_xor(wpop[cb], 32, 64);
            if (hsel == 0) {
                const int cl = 64 * wc + 32 * cb + row_to_channel(j);
                int v = base + 2 * both;
                if constexpr (FUSED) v += thr_lds[cl];
                // y = walked taps + skipped taps
                if constexpr (POS) v -= (s.ks * s.ks - pt.nu * pt.nv) * a.pos.c_in - 2 * skip_lds[cl];
                sub_lds[cl] = FUSED ? (float)v - 0.5f : (float)v;   // exact: multiples of 0.5 below 2^23
            }
        }
        __syncthreads();
        typedef float sub4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const sub4 sb = *reinterpret_cast<const sub4*>(&sub_lds[64 * wc + 32 * cb + 16 * hsel + 4 * q4]);
#pragma unroll
                for (int k = 0; k < 4; ++k) sub[cb][4 * q4 + k] = sb[k];
            }
    }
    if constexpr (FUSED || BRANCH_BITS) {
        // bit = (y >= thr)  <=>  acc - sub = y - thr + 0.5 > 0  <=>  sign bit clear
        // (branch mode: bit = (z >= 0), a real comparison because z may be -0)
        uint32_t* yp = static_cast<uint32_t*>(out);
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            uint32_t part[CB];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                if constexpr (BRANCH) {
                    uint32_t bits = 0;
#pragma unroll
                    for (int r = 0; r < 16; ++r) bits |= (uint32_t)(tot[cb][pb][r] >= 0.0f) << r;
                    part[cb] = bits;
                } else {
                    uint32_t sg = 0;
#pragma unroll
                    for (int r = 15; r >= 0; --r)  // r = 0 ends in bit 0
                        sg = __builtin_amdgcn_alignbit(sg, __float_as_uint(acc[cb][pb][r] - sub[cb][r]), 31);
                    part[cb] = ~sg & 0xFFFFu;     // bit r = (sum >= thr) for channel 16h + r
                }
            }
            // lanes of half 0 finish block 0, lanes of half 1 finish block 1
            const uint32_t give = hsel ? part[0] : part[1];
            const uint32_t got = (uint32_t)__shfl_xor((int)give, 32, 64);
            const uint32_t mine = hsel ? part[1] : part[0];
            uint32_t word = hsel ? (got | (mine << 16)) : (mine | (got << 16));
            int m = m0 + 32 * (PB * wp + pb) + j;
            bool row_ok = m < s.m;
            if constexpr (POS) {
                int n0, oh, ow;
                row_ok = block_pos(PB * wp + pb, n0, oh, ow);
                m = ((n0 + j) * s.ho + oh) * s.wo + ow;
            }
            const int wi = (o0 >> 5) + 2 * wc + hsel;  // packed word index along channels
            if (row_ok && wi < s.cwo) {
                const int valid = s.c_out - 32 * wi;   // real channels in this word
                if (valid < 32) word &= (1u << valid) - 1u;
                yp[(size_t)m * s.cwo + wi] = word;
            }
        }
    } else {
        // int32 sums, or the module's real-valued epilogue.  In registers a lane
        // holds 16 consecutive channels of one pixel, i.e. 64-byte pieces 1 KB
        // apart: poor store granularity.  Each wave therefore transposes its 32
        // pixels x 64 channels of a pixel block through its own 8.5 KB of LDS
        // (the stages are free now); afterwards a lane holds 4 consecutive
        // channels of a pixel, 16 lanes one pixel's 64 channels, and a store
        // instruction writes 256 contiguous bytes per pixel, four pixels at a time.
        constexpr int ROW_WORDS = 64 + 4;                      // padded row: 64 channels
        static_assert(4 * 32 * ROW_WORDS * 4 <= 3 * STAGE_BYTES, "transpose tiles must fit the stages");
        __syncthreads();                                       // every wave is done with the stages
        int32_t* tile = reinterpret_cast<int32_t*>(stage) + wave * (32 * ROW_WORDS);
        const int cgrp = lane & 15;                            // 4-channel group within the wave's 64
        const int prow = lane >> 4;                            // pixel row within a group of four
        const int c0 = o0 + 64 * wc + 4 * cgrp;                // this lane's first channel after the transpose
        const bool vec_ok = (s.c_out % 4 == 0) &&
                            ((reinterpret_cast<uintptr_t>(MODULE ? ep.r : out) & (HALF ? 7 : 15)) == 0) &&
                            (!MODULE || ((reinterpret_cast<uintptr_t>(ep.identity) & (HALF ? 7 : 15)) == 0 &&
                                         ep.id_channels % 4 == 0));
        // per-channel parameters of the lane's four channels (clamped loads for a ragged c_out)
        float pg[4], pb_[4], pa[4], pc[4];
        if constexpr (MODULE) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int ch = c0 + k < s.c_out ? c0 + k : s.c_out - 1;
                pg[k] = BRANCH ? 1.0f : ep.scale[ch];     // branch mode: the sum is already scaled
                pb_[k] = BRANCH ? 0.0f : ep.bias[ch];
                pa[k] = ep.slope ? ep.slope[ch] : 1.0f;
                pc[k] = ep.next_bias ? ep.next_bias[ch] : 0.0f;
            }
        }
        // The identity vectors of a pixel block are fetched one block ahead of
        // their use and before any store of that block: the real stream may be
        // updated in place, so the compiler must not be left to order these
        // loads against the stores, and issued together they overlap.
        real4 ids[AHEAD + 1][8];
        const int id0 = MODULE ? c0 % (ep.id_channels > 0 ? ep.id_channels : 1) : 0;   // channel of the identity stream
        // plain case: descriptors and lane offsets of the three streams (see wave_rows_rsrc)
        const int esz = (int)sizeof(real_t);
        const auto fast_id_res = wave_rows_rsrc(MODULE ? ep.identity : nullptr, ep.id_channels * esz);
        const auto fast_r_res = wave_rows_rsrc(MODULE ? ep.r : nullptr, s.c_out * esz);
        const auto fast_xn_res = wave_rows_rsrc(MODULE ? ep.x_next : nullptr, s.cwo * 4);
        const uint32_t fast_id_off = (uint32_t)((prow * ep.id_channels + id0) * esz);
        const uint32_t fast_r_off = (uint32_t)((prow * s.c_out + c0) * esz);
        const uint32_t fast_xn_off = (cgrp & 7) == 0
            ? (uint32_t)((prow * s.cwo + ((o0 + 64 * wc) >> 5) + (cgrp >> 3)) * 4) : 0x7FFFFFF0u;
        // int32 sums: the same for the output tensor, one offset per channel of the lane
        const auto y_res = wave_rows_rsrc(MODULE ? nullptr : out, s.c_out * 4);
        uint32_t y_off[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) y_off[k] = c0 + k < s.c_out ? (uint32_t)((prow * s.c_out + c0 + k) * 4) : 0x7FFFFFF0u;
        auto load_ids = [&](auto fast_tag, int pb, real4 (&dst)[8]) {
            constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const int m = m0 + 32 * (PB * wp + pb) + 4 * g + prow;
                real4 t4 = {(real_t)0, (real_t)0, (real_t)0, (real_t)0};
                if constexpr (FAST) {
                    t4 = load_real4(fast_id_res, fast_id_off, (32 * pb + 4 * g) * ep.id_channels * (int)sizeof(real_t));
                } else if (ep.identity && m < s.m) {
                    // the identity stream may have fewer channels than the output
                    // (replication by bookkeeping): channel o reads o mod id_channels
                    const real_t* idrow = static_cast<const real_t*>(ep.identity) + (size_t)m * ep.id_channels;
                    if (vec_ok && c0 + 4 <= s.c_out) {      // id_channels % 4 == 0: the four stay together
                        t4 = __builtin_nontemporal_load(reinterpret_cast<const real4*>(idrow + id0));
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (c0 + k < s.c_out) t4[k] = idrow[(id0 + k) % ep.id_channels];
                    }
                }
                dst[g] = t4;
            }
        };
        if constexpr (MODULE && !BRANCH) {
            // the per-channel terms leave the accumulators now, before the identity vectors and the
            // module's parameters occupy registers: sub[][] is dead from here on
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[cb][pb][r] -= sub[cb][r];
            __builtin_amdgcn_sched_barrier(0);
        }
        // FAST: the workgroup tile is whole along the channels, rows are vector
        // aligned and the module has every part (identity, real stream out, next
        // bits): no per-element predicates except the row bound, so the loads and
        // stores of a block issue back to back.  Everything else takes the general path.
        auto run = [&](auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        if constexpr (MODULE) {
#pragma unroll
            for (int k = 0; k < AHEAD && k < PB; ++k) {
                if constexpr (FAST && EARLY_IDS) {
#pragma unroll
                    for (int g = 0; g < 8; ++g) ids[k][g] = early_ids[k][g];     // fetched before the K loop
                } else {
                    load_ids(fast_tag, k, ids[k]);
                }
            }
        }
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; r += 4) {
                    int4 q;
                    if constexpr (BRANCH) {           // float totals travel as their bit patterns
                        q.x = __float_as_int(tot[cb][pb][r + 0]);
                        q.y = __float_as_int(tot[cb][pb][r + 1]);
                        q.z = __float_as_int(tot[cb][pb][r + 2]);
                        q.w = __float_as_int(tot[cb][pb][r + 3]);
                    } else if constexpr (MODULE) {    // the sum is an integer held exactly in a float: it stays one
                        q.x = __float_as_int(acc[cb][pb][r + 0]);
                        q.y = __float_as_int(acc[cb][pb][r + 1]);
                        q.z = __float_as_int(acc[cb][pb][r + 2]);
                        q.w = __float_as_int(acc[cb][pb][r + 3]);
                    } else {
                        q.x = (int)(acc[cb][pb][r + 0] - sub[cb][r + 0]);
                        q.y = (int)(acc[cb][pb][r + 1] - sub[cb][r + 1]);
                        q.z = (int)(acc[cb][pb][r + 2] - sub[cb][r + 2]);
                        q.w = (int)(acc[cb][pb][r + 3] - sub[cb][r + 3]);
                    }
                    *reinterpret_cast<int4*>(tile + j * ROW_WORDS + 32 * cb + 16 * hsel + r) = q;
                }
            if constexpr (MODULE) {
                if (pb + AHEAD < PB) load_ids(fast_tag, pb + AHEAD, ids[(pb + AHEAD) % (AHEAD + 1)]);
            }
            // same wave wrote and reads: LDS operations of a wave complete in order
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const int px = 4 * g + prow;
                const int4 q = *reinterpret_cast<const int4*>(tile + px * ROW_WORDS + 4 * cgrp);
                const int m = m0 + 32 * (PB * wp + pb) + px;
                const bool row_ok = m < s.m;
                if constexpr (!MODULE) {
                    // the sums as a raw buffer per wave (see wave_rows_rsrc): rows past the end and
                    // channels past c_out (offsets set past every size) are dropped by the bounds check
                    const uint32_t row_off = (uint32_t)((32 * pb + 4 * g) * s.c_out * 4);
                    if (vec_ok) {
                        __builtin_amdgcn_raw_buffer_store_b128(v4i{q.x, q.y, q.z, q.w}, y_res, (int)(y_off[0] + row_off), 0, 2);
                    } else {
                        __builtin_amdgcn_raw_buffer_store_b32(q.x, y_res, (int)(y_off[0] + row_off), 0, 2);
                        __builtin_amdgcn_raw_buffer_store_b32(q.y, y_res, (int)(y_off[1] + row_off), 0, 2);
                        __builtin_amdgcn_raw_buffer_store_b32(q.z, y_res, (int)(y_off[2] + row_off), 0, 2);
                        __builtin_amdgcn_raw_buffer_store_b32(q.w, y_res, (int)(y_off[3] + row_off), 0, 2);
                    }
                } else {
                    real_t* rp = static_cast<real_t*>(ep.r) + (size_t)m * s.c_out + c0;
                    const bool whole = FAST || (vec_ok && c0 + 4 <= s.c_out);
                    const int qv[4] = {q.x, q.y, q.z, q.w};
                    float v[4];
                    uint32_t nib = 0;
                    // a missing slope is the slope 1 (pa = 1: 1 * t is t), so FAST always multiplies
                    const bool has_id = FAST || ep.identity != nullptr;
                    const bool has_slope = FAST || ep.slope != nullptr;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if constexpr (BRANCH)
                            v[k] = module_tail<REAL>(__int_as_float(qv[k]), has_id,
                                                     (float)ids[pb % (AHEAD + 1)][g][k], has_slope, pa[k]);
                        else
                            v[k] = module_value<REAL>(__int_as_float(qv[k]), pg[k], pb_[k], has_id,
                                                      (float)ids[pb % (AHEAD + 1)][g][k], has_slope, pa[k]);
                        nib |= (uint32_t)((FAST || c0 + k < s.c_out) && v[k] + pc[k] >= 0.0f) << k;
                    }
                    if constexpr (FAST) {
                        real4 t4;
#pragma unroll
                        for (int k = 0; k < 4; ++k) t4[k] = (real_t)v[k];
                        const int at = (int)(fast_r_off + (uint32_t)((32 * pb + 4 * g) * s.c_out * esz));
                        if constexpr (HALF) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(v2i, t4), fast_r_res, at, 0, 0);
                        else __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, t4), fast_r_res, at, 0, 0);
                    } else if (ep.r && row_ok) {
                        if (whole) {
                            real4 t4;
#pragma unroll
                            for (int k = 0; k < 4; ++k) t4[k] = (real_t)v[k];
                            *reinterpret_cast<real4*>(rp) = t4;
                        } else {
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                if (c0 + k < s.c_out) rp[k] = (real_t)v[k];
                        }
                    }
                    // eight neighbouring lanes hold the 32 channels of one packed word
                    uint32_t wd = nib << (4 * (cgrp & 7));
                    wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
                    wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
                    wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0x141, 0xF, 0xF, true);  // row_half_mirror
                    const int wi = ((o0 + 64 * wc) >> 5) + (cgrp >> 3);
                    if constexpr (FAST) {
                        __builtin_amdgcn_raw_buffer_store_b32(
                            (int)wd, fast_xn_res, (int)(fast_xn_off + (uint32_t)((32 * pb + 4 * g) * s.cwo * 4)), 0, 0);
                    } else if (ep.x_next && row_ok && wi < s.cwo && (cgrp & 7) == 0) {
                        ep.x_next[(size_t)m * s.cwo + wi] = wd;
                    }
                    if constexpr (FAST && !HALF) {     // keeps the live set inside the register budget
                        if (g & 1) __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        };   // run
        if constexpr (PLAIN) {
            run(std::true_type{});
        } else if constexpr (MODULE && BRANCH) {
            if (module_fast) run(std::true_type{});
            else run(std::false_type{});
        } else {
            run(std::false_type{});
        }
    }
}

// Workgroup -> tile.  Consecutive workgroup ids go to different XCDs; give
// each XCD a contiguous range of tiles (channel tile fastest) so that the
// workgroups sharing an input tile share an L2.
__device__ __forceinline__ void decode_tile(const MfmaArgs& a, int& ptile, int& ctile)
{
    int tile = blockIdx.x;
    const int n_tiles = a.n_ptiles * a.n_ctiles;
    const int per_xcd = n_tiles >> 3;
    if (tile < per_xcd * 8) tile = (tile & 7) * per_xcd + (tile >> 3);
    ptile = a.div_ct(tile);
    ctile = tile - ptile * a.n_ctiles;
}

template <int PB, int OUT, bool EVEN, bool PLAIN = false>
__global__ __launch_bounds__(256, ((PB <= 4 && OUT < OUT_BRANCH) ? 2 : 1)) void conv_mfma_fp4_kernel(
    MfmaArgs a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out, ModuleEp ep, BranchEp bp)
{
    __shared__ uint4 stage[stage_units(PB)];
    int ptile, ctile;
    decode_tile(a, ptile, ctile);
    conv_mfma_fp4_tile<PB, OUT, EVEN, PLAIN, false>(a, x, w, thr, out, ep, bp, stage, ptile, ctile, PosTile{});
}

// Position-major tiling of the fused 3x3 convolution, for small feature maps in
// large batches (7 x 7: 40 of 49 windows reach outside the image and 18 % of all
// taps are padding).
//
// The GEMM rows of a tile need not be consecutive pixels: any set of output
// pixels will do, as long as each result is stored where it belongs.  Here a
// pixel block is ONE output position in 32 consecutive images, and the blocks
// are ordered by position class: the interior rectangle (every tap inside the
// image), the top rows, the bottom rows, the left and the right columns.  All
// windows of a class miss the image in the same filter rows or columns, so a
// tile of one class walks only the taps of that class's rectangle (6 of 9 for
// an edge) and accounts for the others in closed form: a tap outside the image
// reads -1 in every channel, so its dot product with the weights is
// c_in - 2 * popcount(weight words of that tap), one number per output channel,
// counted when the workgroup starts.  A corner shares the tile of its edge row:
// the tap columns it misses on top of the row's are read as zero words, as in
// the pixel-major kernel.
//
// The classes also level the work: interior tiles (9 taps) take PBI pixel
// blocks per wave, edge tiles (6 taps) PBE > PBI, chosen by the launcher so
// that every tile of the launch gets its own CU and the longest tile is as
// short as possible (7 x 7 map, 256 images, 1024 channels: 160 tiles of 10
// blocks x 9 taps and 96 tiles of 16 blocks x 6 taps on 256 CUs, against 224
// tiles of 14 blocks x 9 taps pixel-major).  One kernel holds both tile bodies
// and a workgroup picks its own.
template <int PBI, int PBE, int NW>
__global__ __launch_bounds__(64 * NW, 1) void conv_mfma_fp4_pos_kernel(
    MfmaArgs a, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, uint32_t* __restrict__ out)
{
    __shared__ uint4 stage[stage_units(PBI > PBE ? PBI : PBE, NW)];
    int ptile, ctile;
    decode_tile(a, ptile, ctile);
    const PosTile pt = pos_tile(a.pos, ptile, NW / 2);   // segment table -> this workgroup's tile (wave-uniform selects)
    const ModuleEp ep{};
    const BranchEp bp{};
    if (PBI != PBE && pt.pb == PBI)
        conv_mfma_fp4_tile<PBI, OUT_BITS, true, false, true, NW>(a, x, w, thr, out, ep, bp, stage, ptile, ctile, pt);
    else
        conv_mfma_fp4_tile<PBE, OUT_BITS, true, false, true, NW>(a, x, w, thr, out, ep, bp, stage, ptile, ctile, pt);
}

template <int PB, int OUT>
hipError_t launch_pb(MfmaArgs a, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                     void* out, const ModuleEp* ep, hipStream_t stream, const BranchEp* bp = nullptr)
{
    const ModuleEp e = ep ? *ep : ModuleEp{};
    const BranchEp b = bp ? *bp : BranchEp{};
    constexpr int WG_PX = 64 * PB;
    a.n_ptiles = (a.s.m + WG_PX - 1) / WG_PX;
    a.div_ct = DivBy::make(a.n_ctiles);
    const unsigned blocks = (unsigned)(a.n_ptiles * a.n_ctiles);
    if constexpr (OUT >= OUT_MODULE_F32 && OUT <= OUT_MODULE_BF16) {
        // the plain case of a module call (see the kernel's PLAIN parameter)
        const uintptr_t al = OUT == OUT_MODULE_F32 ? 15 : 7;
        // (c_out bound: a wave's rows of any of the three streams stay below 2^31 bytes)
        const bool plain = e.identity && e.r && e.x_next && a.s.c_out % WG_CH == 0 && e.id_channels % 4 == 0 &&
                           a.s.c_out <= (1 << 20) &&
                           ((reinterpret_cast<uintptr_t>(e.r) | reinterpret_cast<uintptr_t>(e.identity)) & al) == 0;
        if (plain) {
            if (a.units_per_tap % 2 == 0)
                hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, OUT, true, true>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out, e, b);
            else
                hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, OUT, false, true>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out, e, b);
            return hipGetLastError();
        }
    }
    if constexpr (OUT >= OUT_BRANCH) {
        hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, OUT, true>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out, e, b);
    } else {
        if (a.units_per_tap % 2 == 0)
            hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, OUT, true>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out, e, b);
        else
            hipLaunchKernelGGL((conv_mfma_fp4_kernel<PB, OUT, false>), dim3(blocks), dim3(256), 0, stream, a, x, w, thr, out, e, b);
    }
    return hipGetLastError();
}

}  // namespace

// Branch-mode launchers, one translation unit per pad mode (the kernel is big;
// this keeps the build parallel).  kind: KIND_* of the header's enum.
hipError_t launch_branch_mfma_pad_minus(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                        hipStream_t stream);
hipError_t launch_branch_mfma_pad_words(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                        hipStream_t stream);
hipError_t launch_branch_mfma_pad_skip(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                       hipStream_t stream);

// Shared body of those three.
template <int PADMODE>
hipError_t launch_branch_mfma_kind(const MfmaArgs& a, const BranchArgs& b, const BranchEp& bp, int kind,
                                   hipStream_t stream)
{
    switch (kind) {
        case KIND_F32:
            return launch_pb<4, OUT_BRANCH + 4 * PADMODE + KIND_F32>(a, b.x, b.w, nullptr, b.out, b.tail, stream, &bp);
        case KIND_BITS:
            return launch_pb<4, OUT_BRANCH + 4 * PADMODE + KIND_BITS>(a, b.x, b.w, nullptr, b.out, b.tail, stream, &bp);
        case KIND_TAIL_F32:
            return launch_pb<4, OUT_BRANCH + 4 * PADMODE + KIND_TAIL_F32>(a, b.x, b.w, nullptr, b.out, b.tail, stream, &bp);
        case KIND_TAIL_F16:
            return launch_pb<4, OUT_BRANCH + 4 * PADMODE + KIND_TAIL_F16>(a, b.x, b.w, nullptr, b.out, b.tail, stream, &bp);
        default:
            return hipErrorInvalidValue;
    }
}

}  // namespace bcnn
