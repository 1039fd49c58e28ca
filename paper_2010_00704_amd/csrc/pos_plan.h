// Position-major tiling of the fused 3x3 convolution: the plan the host makes and the arithmetic
// that turns a tile index into output positions.  Plain C++ on purpose: the launcher fills the
// plan, the kernel decodes it, and a host-only test walks every tile of many shapes through the
// same functions and checks that each output pixel is produced exactly once and that no tap
// which a tile leaves out is inside the image for any of its pixels.
//
// A pixel block (32 GEMM rows) is one output position in 32 consecutive images.  Positions fall
// into five rectangles (segments): the interior (every tap of every window inside the image), the
// top rows, the bottom rows (both with their corners), the left and the right columns.  All windows
// of a segment miss the image in the same filter rows or columns, so its tiles walk the taps of one
// rectangle u_lo .. u_lo+nu-1 x v_lo .. v_lo+nv-1 only.  Blocks of a segment are numbered position
// by position (row by row inside the rectangle), image groups fastest, and cut into tiles of
// (waves along the pixels) * pb blocks.
#pragma once
#include "div_by.h"

// (always inlined on the device: the plan sits in the kernel arguments, and a call that is not
// inlined would copy it to private memory first)
#if defined(__HIPCC__)
#define BCNN_PLAN_INLINE __host__ __device__ __forceinline__
#else
#define BCNN_PLAN_INLINE inline
#endif

namespace bcnn {

struct PosSeg {
    int32_t tile0;      // first tile (per channel tile) of the segment
    int32_t blocks;     // pixel blocks of the segment = positions * groups of 32 images
    int32_t oh0, ow0, width;   // the rectangle's corner and width
    int32_t u_lo, nu, v_lo, nv; // filter rows / columns that some window of the segment has inside the image
    int32_t pb;         // pixel blocks per wave of the segment's tiles
    DivBy div_width;
};
struct PosArgs {
    PosSeg seg[5];
    int32_t groups;     // n / 32
    DivBy div_groups;
    int32_t z_per_tap;  // 32 * cw - c_in: channel-tail positions of one tap (zero on both sides)
    int32_t c_in;
    DivBy div_per_tap;  // by cw / 4, the 16-byte units of a tap
};
// One workgroup's tile.
struct PosTile {
    int32_t block0;     // first block of the tile within its segment
    int32_t blocks;     // blocks of the segment
    int32_t oh0, ow0, width;
    int32_t u_lo, nu, v_lo, nv;
    int32_t pb;
    DivBy div_width;
};

// Tile `ptile` (within a channel tile) of the plan, for workgroups with `wp` waves along the pixels.
BCNN_PLAN_INLINE PosTile pos_tile(const PosArgs& p, int ptile, int wp)
{
    // (field by field, with constant indices: the table lives in the kernel arguments; copying a
    // whole entry chosen at run time makes the compiler select between addresses, and then the
    // argument block is copied to private memory first)
    const int k = (ptile >= p.seg[1].tile0 ? 1 : 0) + (ptile >= p.seg[2].tile0 ? 1 : 0) +
                  (ptile >= p.seg[3].tile0 ? 1 : 0) + (ptile >= p.seg[4].tile0 ? 1 : 0);
#define BCNN_POS_PICK(f) \
    (k == 4 ? p.seg[4].f : k == 3 ? p.seg[3].f : k == 2 ? p.seg[2].f : k == 1 ? p.seg[1].f : p.seg[0].f)
    PosTile t;
    t.pb = BCNN_POS_PICK(pb);
    t.block0 = (ptile - BCNN_POS_PICK(tile0)) * wp * t.pb;
    t.blocks = BCNN_POS_PICK(blocks);
    t.oh0 = BCNN_POS_PICK(oh0);
    t.ow0 = BCNN_POS_PICK(ow0);
    t.width = BCNN_POS_PICK(width);
    t.u_lo = BCNN_POS_PICK(u_lo);
    t.nu = BCNN_POS_PICK(nu);
    t.v_lo = BCNN_POS_PICK(v_lo);
    t.nv = BCNN_POS_PICK(nv);
    t.div_width.mul = BCNN_POS_PICK(div_width.mul);
    t.div_width.shift = BCNN_POS_PICK(div_width.shift);
    t.div_width.d = BCNN_POS_PICK(div_width.d);
#undef BCNN_POS_PICK
    return t;
}

// Block `bl` of a tile -> first image and output position; false past the segment's end (the last
// block's numbers are returned then).
BCNN_PLAN_INLINE bool pos_block(const PosArgs& p, const PosTile& t, int bl, int& n0, int& oh, int& ow)
{
    const int bidx = t.block0 + bl;
    const bool active = bidx < t.blocks;
    const int bc = active ? bidx : t.blocks - 1;
    const int pi = p.div_groups(bc);
    n0 = 32 * (bc - pi * p.groups);
    const int q = t.div_width(pi);
    oh = t.oh0 + q;
    ow = t.ow0 + (pi - q * t.width);
    return active;
}

// ---- the plan (host)
// Taps of a 3-tap axis that are inside the image for output index o: [lo, hi] within 0..2.
inline void pos_axis_taps(int o, int stride, int pad, int extent, int& lo, int& hi)
{
    const int p = o * stride - pad;
    lo = p < 0 ? -p : 0;
    hi = p + 2 >= extent ? extent - 1 - p : 2;
}
// Splits 0..count-1 into leading indices that miss taps at the low end, a middle with all three taps
// and trailing indices that miss taps at the high end; false if that is not the structure.
inline bool pos_axis_classes(int count, int stride, int pad, int extent, int& first_full, int& end_full,
                             int& lead_lo, int& trail_hi)
{
    first_full = 0;
    lead_lo = 0;
    trail_hi = 2;
    int lo, hi;
    while (first_full < count) {
        pos_axis_taps(first_full, stride, pad, extent, lo, hi);
        if (lo == 0) break;
        if (hi < 2 || lo > 2) return false;
        lead_lo = first_full == 0 ? lo : (lo < lead_lo ? lo : lead_lo);
        ++first_full;
    }
    end_full = first_full;
    while (end_full < count) {
        pos_axis_taps(end_full, stride, pad, extent, lo, hi);
        if (lo != 0) return false;
        if (hi < 2) break;
        ++end_full;
    }
    for (int o = end_full; o < count; ++o) {
        pos_axis_taps(o, stride, pad, extent, lo, hi);
        if (lo != 0 || hi < 0) return false;
        trail_hi = o == end_full ? hi : (hi > trail_hi ? hi : trail_hi);
    }
    if (end_full == count) trail_hi = 2;
    return true;
}

struct PosShape { int32_t n, h, w, cw, c_in, ks, stride, pad, ho, wo; };

// Fills `p` for workgroups of nw waves, interior tiles of pbi blocks per wave and edge tiles of pbe.
// Returns the tiles per channel tile, or -1 if the shape does not fit the scheme; *longest = the
// most (taps walked) x (blocks per wave) of any tile.
inline int pos_plan(const PosShape& s, int pbi, int pbe, int nw, PosArgs& p, int* longest)
{
    if (s.ks != 3 || s.cw % 8 != 0 || s.n % 32 != 0 || s.n <= 0 || s.ho > 1023 || s.wo > 1023) return -1;
    int r0, r1, c0, c1, top_lo, bottom_hi, left_lo, right_hi;
    if (!pos_axis_classes(s.ho, s.stride, s.pad, s.h, r0, r1, top_lo, bottom_hi)) return -1;
    if (!pos_axis_classes(s.wo, s.stride, s.pad, s.w, c0, c1, left_lo, right_hi)) return -1;
    p.groups = s.n / 32;
    p.div_groups = DivBy::make(p.groups);
    p.c_in = s.c_in;
    p.z_per_tap = 32 * s.cw - p.c_in;
    p.div_per_tap = DivBy::make(s.cw / 4);
    struct Rect { int oh0, rows, ow0, cols, u_lo, nu, v_lo, nv; };
    const Rect rects[5] = {
        {r0, r1 - r0, c0, c1 - c0, 0, 3, 0, 3},                         // interior
        {0, r0, 0, s.wo, top_lo, 3 - top_lo, 0, 3},                     // top rows, corners included
        {r1, s.ho - r1, 0, s.wo, 0, bottom_hi + 1, 0, 3},               // bottom rows, corners included
        {r0, r1 - r0, 0, c0, 0, 3, left_lo, 3 - left_lo},               // left columns
        {r0, r1 - r0, c1, s.wo - c1, 0, 3, 0, right_hi + 1},            // right columns
    };
    int tiles = 0;
    *longest = 0;
    for (int i = 0; i < 5; ++i) {
        const Rect& r = rects[i];
        PosSeg& g = p.seg[i];
        g.tile0 = tiles;
        g.blocks = r.rows * r.cols * p.groups;
        g.oh0 = r.oh0; g.ow0 = r.ow0; g.width = r.cols > 0 ? r.cols : 1;
        g.u_lo = r.u_lo; g.nu = r.nu; g.v_lo = r.v_lo; g.nv = r.nv;
        g.pb = i == 0 ? pbi : pbe;
        g.div_width = DivBy::make(g.width);
        const int per_tile = (nw / 2) * g.pb;
        const int n = (g.blocks + per_tile - 1) / per_tile;
        tiles += n;
        if (n > 0 && r.nu * r.nv * g.pb > *longest) *longest = r.nu * r.nv * g.pb;
    }
    return tiles;
}

}  // namespace bcnn
