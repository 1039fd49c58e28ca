// Launchers of the matrix-core convolution (kernel: conv_mfma_fp4_kernel.h).
#include "conv_mfma_fp4_kernel.h"

namespace bcnn {

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
    // and a wave's rows of an output tensor (up to 224 rows of c_out 4-byte elements) by 31-bit offsets too
    return s.cw % 4 == 0 && (bits & 15) == 0 && 256 * n_chunks + s.k + 2 < (1 << 22) &&
           x_bytes < (1ll << 31) && w_bytes < (1ll << 31) && s.c_out <= (1 << 20);
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

// ---- position-major tiling (kernel: conv_mfma_fp4_pos_kernel; plan: pos_plan.h)
// Fills a.pos and a.n_ptiles for workgroups of nw waves, interior tiles of pbi blocks per wave and
// edge tiles of pbe.  Returns the cost in the units of tile_cost() times taps (rounds of workgroups
// x the longest tile), or a negative number if the shape does not fit the scheme.
static double plan_pos(const ConvShape& s, int pbi, int pbe, int nw, MfmaArgs& a)
{
    const PosShape ps = {s.n, s.h, s.w, s.cw, s.ks > 0 ? s.k / (s.ks * s.ks) : 0, s.ks, s.stride, s.pad, s.ho, s.wo};
    int longest = 0;
    const int tiles = pos_plan(ps, pbi, pbe, nw, a.pos, &longest);
    if (tiles < 0) return -1.0;
    a.n_ptiles = tiles;
    const int64_t wgs = (int64_t)tiles * a.n_ctiles;
    const int64_t resident = 256 * (4 / nw);     // one wave per SIMD
    return (double)((wgs + resident - 1) / resident) * longest;
}

bool conv_mfma_fp4_pos_supported(const ConvShape& s)
{
    MfmaArgs a;
    a.n_ctiles = (s.c_out + WG_CH - 1) / WG_CH;
    return plan_pos(s, 7, 7, 4, a) > 0.0;
}

// (interior, edge) pixel blocks per wave the position-major kernel is built for, as tile codes
// 10 * pbi + pbe; and the waves per workgroup of each
static const int POS_TILES[] = {58, 68, 67, 77};
static int pos_waves(int code) { return code == 58 || code == 68 ? 2 : 4; }

static hipError_t launch_pos(MfmaArgs& a, int code, const uint32_t* x, const uint32_t* w, const int32_t* thr, void* out,
                             hipStream_t stream)
{
    a.div_ct = DivBy::make(a.n_ctiles);
    const dim3 blocks((unsigned)(a.n_ptiles * a.n_ctiles));
    uint32_t* y = static_cast<uint32_t*>(out);
    switch (code) {
        case 58: hipLaunchKernelGGL((conv_mfma_fp4_pos_kernel<5, 8, 2>), blocks, dim3(128), 0, stream, a, x, w, thr, y); break;
        case 68: hipLaunchKernelGGL((conv_mfma_fp4_pos_kernel<6, 8, 2>), blocks, dim3(128), 0, stream, a, x, w, thr, y); break;
        case 67: hipLaunchKernelGGL((conv_mfma_fp4_pos_kernel<6, 7, 4>), blocks, dim3(256), 0, stream, a, x, w, thr, y); break;
        case 77: hipLaunchKernelGGL((conv_mfma_fp4_pos_kernel<7, 7, 4>), blocks, dim3(256), 0, stream, a, x, w, thr, y); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_conv_mfma_fp4(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                                const int32_t* thr, void* out, const ModuleEp* ep, int tile,
                                hipStream_t stream)
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
    a.row_jump = (s.w - s.ks) * s.cw;
    a.tap_step = 0;
    a.taps = s.ks * s.ks;
    a.chunks_per_tap = 0;
    a.div_hw = DivBy::make(s.ho * s.wo);
    a.div_wo = DivBy::make(s.wo);
    // Feature maps of 7, 14, 28, 56 pixels a side make the pixel count a
    // multiple of 49: 7 pixel blocks per wave then tile it without remainder
    // where 4 would leave a quarter of the last round idle.  The 2 x 7 tile
    // runs one workgroup per CU, so nothing hides its prologue and epilogue,
    // where two co-resident 2 x 4 workgroups per CU overlap each other's ends.
    // Measured where the wide tile saves a round, on launches whose 2 x 4
    // workgroups are all resident at once (392 of them): 7-9 % ahead at 14 to
    // 36 chunks, 2-3 % at 9, level at 4, behind at 3; with 784 workgroups and 9
    // chunks the two tiles are level, so there the narrow one stays up to 16
    // chunks; where the wide tile saves no round the narrow one wins at every
    // length.  Only the fused kernel has the
    // registers for it: the int32 epilogue of a 2 x 7 tile would spill.
    // `tile` = 4 or 7 forces a tile (for tests and measurements), 0 chooses.
    if (ep && ep->half == REAL_BF16) return launch_pb<4, OUT_MODULE_BF16>(a, x, w, nullptr, nullptr, ep, stream);
    if (ep && ep->half) return launch_pb<4, OUT_MODULE_F16>(a, x, w, nullptr, nullptr, ep, stream);
    if (ep) return launch_pb<4, OUT_MODULE_F32>(a, x, w, nullptr, nullptr, ep, stream);
    if (!thr) return launch_pb<4, OUT_I32>(a, x, w, thr, out, nullptr, stream);
    // `tile` = 58, 67 or 77: position-major tiles of that (interior, edge) width, forced.
    if (tile > 10) {
        if (plan_pos(s, tile / 10, tile % 10, pos_waves(tile), a) < 0.0) return hipErrorInvalidValue;
        return launch_pos(a, tile, x, w, thr, out, stream);
    }
    const int64_t wgs4 = ((s.m + 255) / 256) * a.n_ctiles;     // workgroups of the 2 x 4 tile; 512 are resident at once
    const bool long_enough = a.n_chunks >= 16 || (a.n_chunks >= 9 && wgs4 <= 512);
    const bool wide = tile == 7 || (tile == 0 && long_enough && tile_cost(s, 7) < tile_cost(s, 4));
    // Position-major tiles where they shorten the longest workgroup by a tenth or more against the
    // better of the two pixel-major tiles (they walk fewer taps on the edges and level the rest;
    // their set-up is longer), and only where a pixel's channels fill whole 128-byte lines: the rows
    // of a position-major block lie a whole image apart, so with fewer channels every 32-byte piece
    // a chunk needs costs a line of its own (measured: 28 x 28 map with 256 channels, 21 us against
    // 18 us).  Measured over 7 x 7 to 28 x 28 maps, 512 to 2048 channels and 32 to 512 images, the
    // choice is within 4 % of the best forced variant.
    if (tile == 0 && s.cw >= 32) {
        const double plain = (wide ? tile_cost(s, 7) : tile_cost(s, 4)) * 9.0;
        double best = 0.9 * plain;
        int best_code = 0;
        for (const int code : POS_TILES) {
            MfmaArgs ap = a;
            const double cost = plan_pos(s, code / 10, code % 10, pos_waves(code), ap);
            if (cost > 0.0 && cost < best) { best = cost; best_code = code; }
        }
        if (best_code) {
            plan_pos(s, best_code / 10, best_code % 10, pos_waves(best_code), a);
            return launch_pos(a, best_code, x, w, thr, out, stream);
        }
    }
    if (wide) return launch_pb<7, OUT_BITS>(a, x, w, thr, out, nullptr, stream);
    return launch_pb<4, OUT_BITS>(a, x, w, thr, out, nullptr, stream);
}

// ---- branch mode on the matrix cores
static int64_t branch_x_bytes(const ConvShape& s, const BranchArgs& b)
{
    const int64_t one = (int64_t)s.n * s.h * s.w * s.cw * 4;
    return b.x_branch_stride ? (int64_t)(b.branches - 1) * b.x_branch_stride * 4 + one : one;
}

bool conv_branches_mfma_supported(const ConvShape& s, const BranchArgs& b)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(b.x) | reinterpret_cast<uintptr_t>(b.w) |
                           ((uintptr_t)b.x_branch_stride * 4u);
    const int64_t w_bytes = (int64_t)s.c_out * b.branches * s.cw * 4;
    // whole 256-bit chunks per branch, 16-byte aligned tensors, pad words that fit
    // the LDS table, validity masks of 32 bits, 31-bit byte offsets
    return s.cw % 8 == 0 && (bits & 15) == 0 && (int64_t)b.branches * s.cw <= PAD_LDS_WORDS &&
           b.branches <= MAX_BRANCHES && branch_x_bytes(s, b) < (1ll << 31) && w_bytes < (1ll << 31);
}

hipError_t launch_conv_branches_mfma(const ConvShape& s, const BranchArgs& b, hipStream_t stream)
{
    MfmaArgs a;
    a.s = s;
    a.n_ptiles = 0;
    a.n_ctiles = (s.c_out + WG_CH - 1) / WG_CH;
    a.units_per_tap = s.cw / 4;
    a.taps = b.branches;
    a.n_units = a.taps * a.units_per_tap;
    a.n_chunks = a.n_units / 2;
    a.chunks_per_tap = s.cw / 8;
    a.z = 0;
    a.x_bytes = (int32_t)branch_x_bytes(s, b);
    a.w_bytes = (int32_t)((int64_t)s.c_out * a.n_units * 16);
    // 3x3: the input offset walks on through the taps of a filter row and jumps at
    // its end; 1x1 with parallel branches: every branch starts at the same pixel
    a.row_jump = s.ks == 1 ? 0 : (s.w - s.ks) * s.cw;
    a.tap_step = (int32_t)b.x_branch_stride + (s.ks == 1 ? -s.cw : 0);
    a.div_hw = DivBy::make(s.ho * s.wo);
    a.div_wo = DivBy::make(s.wo);
    BranchEp bp;
    bp.scale = b.scale;
    bp.bias = b.bias;
    bp.pad_words = b.pad_words;
    bp.pad_mode = b.zero_pad ? 2 : (b.pad_words ? 1 : 0);
    const int kind = b.tail ? (b.tail->half ? KIND_TAIL_F16 : KIND_TAIL_F32) : (b.fused ? KIND_BITS : KIND_F32);
    if (bp.pad_mode == 2) return launch_branch_mfma_pad_skip(a, b, bp, kind, stream);
    if (bp.pad_mode == 1) return launch_branch_mfma_pad_words(a, b, bp, kind, stream);
    return launch_branch_mfma_pad_minus(a, b, bp, kind, stream);
}

}  // namespace bcnn
