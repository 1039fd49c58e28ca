// Host-only check of the position-major tiling plan (csrc/pos_plan.h): for a grid of shapes and every
// tile width the kernel is built for, walk every tile of the plan through the same decode functions
// the kernel uses and check that
//   - every output pixel (image, oh, ow) is produced by exactly one active row of one tile,
//   - every filter tap a tile does not walk lies outside the image for every pixel of the tile
//     (so replacing it by "-1 in every channel" is right),
//   - every tap that is inside the image for a pixel is walked by its tile,
//   - the tile count matches, and shapes outside the scheme are refused.
// Prints "mismatches: N"; exit status 0 = none.
#include "pos_plan.h"

#include <cstdio>
#include <vector>

using namespace bcnn;

static long check_shape(int n, int h, int w, int stride, int pad, int pbi, int pbe, int nw, long* planned)
{
    PosShape s;
    s.n = n; s.h = h; s.w = w; s.cw = 8; s.c_in = 250; s.ks = 3; s.stride = stride; s.pad = pad;
    s.ho = (h + 2 * pad - 3) / stride + 1;
    s.wo = (w + 2 * pad - 3) / stride + 1;
    if (s.ho < 1 || s.wo < 1) return 0;
    PosArgs p;
    int longest = 0;
    const int tiles = pos_plan(s, pbi, pbe, nw, p, &longest);
    if (tiles < 0) return 0;
    ++*planned;
    long bad = 0;
    const int wp = nw / 2;
    std::vector<int> seen((size_t)n * s.ho * s.wo, 0);
    int most = 0;
    for (int t = 0; t < tiles; ++t) {
        const PosTile pt = pos_tile(p, t, wp);
        if (pt.nu * pt.nv * pt.pb > most) most = pt.nu * pt.nv * pt.pb;
        if (pt.u_lo < 0 || pt.nu < 1 || pt.u_lo + pt.nu > 3 || pt.v_lo < 0 || pt.nv < 1 || pt.v_lo + pt.nv > 3) ++bad;
        int active_blocks = 0;
        for (int bl = 0; bl < wp * pt.pb; ++bl) {
            int n0, oh, ow;
            const bool active = pos_block(p, pt, bl, n0, oh, ow);
            if (n0 < 0 || n0 + 32 > n || oh < 0 || oh >= s.ho || ow < 0 || ow >= s.wo) { ++bad; continue; }
            if (!active) continue;
            ++active_blocks;
            for (int j = 0; j < 32; ++j) seen[((size_t)(n0 + j) * s.ho + oh) * s.wo + ow] += 1;
            for (int u = 0; u < 3; ++u)
                for (int v = 0; v < 3; ++v) {
                    const int ih = oh * stride - pad + u, iw = ow * stride - pad + v;
                    const bool inside = ih >= 0 && ih < h && iw >= 0 && iw < w;
                    const bool walked = u >= pt.u_lo && u < pt.u_lo + pt.nu && v >= pt.v_lo && v < pt.v_lo + pt.nv;
                    if (inside && !walked) ++bad;   // a tap with real data would be replaced by padding
                }
        }
        if (active_blocks == 0) ++bad;              // an empty tile
    }
    for (int c : seen)
        if (c != 1) ++bad;
    if (most != longest) ++bad;
    return bad;
}

int main()
{
    long bad = 0, planned = 0;
    const int widths[][3] = {{5, 8, 2}, {6, 8, 2}, {6, 7, 4}, {7, 7, 4}};
    for (const auto& wd : widths)
        for (int n : {32, 64, 160})
            for (int h = 1; h <= 19; ++h)
                for (int w = 1; w <= 19; w += (h % 3 == 0 ? 1 : 2))
                    for (int stride = 1; stride <= 2; ++stride)
                        for (int pad = 0; pad <= 2; ++pad)   // (pad 2: two rows miss taps at the top, unequally)
                            bad += check_shape(n, h, w, stride, pad, wd[0], wd[1], wd[2], &planned);
    // the benchmark shapes with a 3 x 3 filter
    bad += check_shape(256, 7, 7, 1, 1, 5, 8, 2, &planned);
    bad += check_shape(64, 28, 28, 1, 1, 6, 8, 2, &planned);
    bad += check_shape(64, 56, 56, 2, 1, 6, 7, 4, &planned);
    // what the scheme does not cover
    {
        PosArgs p;
        int longest;
        PosShape s = {32, 7, 7, 8, 256, 3, 1, 1, 7, 7};
        PosShape t = s; t.n = 31; if (pos_plan(t, 7, 7, 4, p, &longest) >= 0) ++bad;      // not whole groups of 32 images
        t = s; t.cw = 4; if (pos_plan(t, 7, 7, 4, p, &longest) >= 0) ++bad;               // chunks would straddle taps
        t = s; t.ks = 1; if (pos_plan(t, 7, 7, 4, p, &longest) >= 0) ++bad;
        t = s; t.h = 1; t.ho = 1; if (pos_plan(t, 7, 7, 4, p, &longest) >= 0) ++bad;       // one row misses taps on both sides
        if (pos_plan(s, 7, 7, 4, p, &longest) != 2 + 1 + 1 + 1 + 1) ++bad;                // 25, 7, 7, 5, 5 blocks in tiles of 14
        if (longest != 63) ++bad;
    }
    if (planned < 2000) ++bad;
    printf("planned shapes: %ld\nmismatches: %ld\n", planned, bad);
    return bad ? 1 : 0;
}
