// Parallel binary 1x1 branches, each with its own real scale per output channel,
// summed (BCNN paper, Figure 2 bottom), and the F x F binary convolution built
// from F*F such branches on shifted copies of the map (Section 4.2.1, last
// paragraph):
//   y_t = sum_c X_t[shifted by tap t][c] * W[o][t][c]        (integer, |y_t| <= c_in)
//   z   = bias[o] + sum_t scale[t][o] * y_t                  (float)
// evaluated as z = bias[o]; z = fma(scale[t][o], float(y_t), z) for t = 0, 1, ...
// so that the result does not depend on the tiling.
//
// The kernel is the tap-outer xor/popcount loop of the vector-ALU convolution:
// a wave owns 64*TM output pixels (lanes) x 32 output channels; the weights, the
// scales and the pad words are wave-uniform and are read with scalar loads.
// Per tap the popcounts of that tap alone are accumulated (c_in/32 words), then
// folded into the float sums with one integer multiply-add, one conversion and
// one fused multiply-add per (pixel, channel).  A tap outside the image is, per
// mode, the all-zero word (-1 everywhere), the branch's pad words (the sign of
// the branch's bias per channel: the paper zero-fills before the bias), or
// skipped altogether (a contribution of exactly 0).
#include "valu_epilogue.h"

namespace bcnn {
namespace {

using valu::TN;
enum { PAD_MINUS = 0, PAD_WORDS = 1, PAD_SKIP = 2 };
enum { OUT_F32 = 0, OUT_BITS = 1, OUT_TAIL_F32 = 2, OUT_TAIL_F16 = 3 };   // what happens to the branch sum

template <int TM, int VEC, int PADMODE, int OUT, bool FULL>
__global__ __launch_bounds__(256) void conv_branches_kernel(
    ConvShape s, int32_t taps, int32_t n_mtiles, int32_t n_ctiles,
    const uint32_t* __restrict__ x, int64_t x_branch_stride, const uint32_t* __restrict__ w,
    const uint32_t* __restrict__ pad_words, const float* __restrict__ scale,
    const float* __restrict__ bias, void* __restrict__ out, ModuleEp ep)
{
    constexpr bool FUSED = OUT == OUT_BITS;
    static_assert(OUT < OUT_TAIL_F32 || FULL, "the module tail is built for full channel tiles");
    // full tiles with float or real outputs leave through a per-wave LDS tile (valu_epilogue.h)
    constexpr bool WAVE_EPILOGUE = FULL && OUT != OUT_BITS;
    __shared__ uint32_t ep_tile[WAVE_EPILOGUE ? 4 * 64 * valu::TROW : 1];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + wave;
    const int ctile = tile % n_ctiles;
    const int mtile = tile / n_ctiles;
    if (mtile >= n_mtiles) return;
    // FULL (c_out >= 32): every tile computes 32 real channels.  The last tile of
    // a ragged c_out starts at c_out - 32 instead of 32*ctile and drops the
    // `shift` channels it shares with its neighbour when it stores, so no index
    // is ever clamped.  Otherwise (c_out < 32) rows of channels beyond c_out are
    // clamped to the last real one so that every scalar load stays inside its
    // tensor.
    const int o_last = s.c_out - 1;
    const int o0 = (FULL && ctile * TN + TN > s.c_out) ? s.c_out - TN : ctile * TN;
    const int shift = ctile * TN - o0;
    auto chan = [&](int o) -> uint32_t {
        if constexpr (FULL) return (uint32_t)(o0 + o);
        else return (uint32_t)((o0 + o < o_last) ? (o0 + o) : o_last);
    };

    int pn[TM], ph[TM], pw[TM];
    bool live[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = mtile * (64 * TM) + i * 64 + lane;
        live[i] = m < s.m;
        const int mc = live[i] ? m : s.m - 1;
        const int hw = s.ho * s.wo;
        pn[i] = mc / hw;
        const int r = mc - pn[i] * hw;
        const int oh = r / s.wo;
        ph[i] = oh * s.stride - s.pad;
        pw[i] = (r - oh * s.wo) * s.stride - s.pad;
    }

    float z[TM][TN];
    if (bias) {
        const float* bp = bias + (FULL ? o0 : 0);
#pragma unroll
        for (int o = 0; o < TN; ++o) {
            float b;
            if constexpr (FULL) b = bp[o];
            else b = bias[chan(o)];
#pragma unroll
            for (int i = 0; i < TM; ++i) z[i][o] = b;
        }
    } else {
#pragma unroll
        for (int o = 0; o < TN; ++o)
#pragma unroll
            for (int i = 0; i < TM; ++i) z[i][o] = 0.0f;
    }

    // taps = branches: ks*ks shifted ones, or any number of unshifted ones when ks == 1
    const int c_in = s.k / (s.ks * s.ks);  // real channels: the K of one branch
    const uint32_t wrow = (uint32_t)(taps * s.cw);

    for (int tap = 0; tap < taps; ++tap) {
        const int u = s.ks == 1 ? 0 : tap / s.ks, v = s.ks == 1 ? 0 : tap - u * s.ks;
        const uint32_t* xt = x + (size_t)tap * (size_t)x_branch_stride;
        const uint32_t* xp[TM];
        bool inb[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int ih = ph[i] + u, iw = pw[i] + v;
            inb[i] = ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            const int ihc = inb[i] ? ih : 0, iwc = inb[i] ? iw : 0;
            xp[i] = xt + ((size_t)(pn[i] * s.h + ihc) * s.w + iwc) * s.cw;
        }
        int32_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int o = 0; o < TN; ++o) acc[i][o] = 0;

        const uint32_t* wt = w + (uint32_t)(tap * s.cw);
        for (int j0 = 0; j0 < s.cw; j0 += VEC) {
            uint32_t pwv[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) pwv[j] = 0u;
            if constexpr (PADMODE == PAD_WORDS) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) pwv[j] = pad_words[(size_t)tap * s.cw + j0 + j];
            }
            uint32_t xv[TM][VEC];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if constexpr (VEC == 1) {
                    xv[i][0] = inb[i] ? xp[i][j0] : pwv[0];
                } else if constexpr (VEC == 2) {
                    const uint2 t = inb[i] ? *reinterpret_cast<const uint2*>(xp[i] + j0) : make_uint2(pwv[0], pwv[1]);
                    xv[i][0] = t.x; xv[i][1] = t.y;
                } else {
                    const uint4 t = inb[i] ? *reinterpret_cast<const uint4*>(xp[i] + j0)
                                           : make_uint4(pwv[0], pwv[1], pwv[2], pwv[3]);
                    xv[i][0] = t.x; xv[i][1] = t.y; xv[i][2] = t.z; xv[i][3] = t.w;
                }
            }
#pragma unroll
            for (int o = 0; o < TN; ++o) {
                const uint32_t* wp = wt + (chan(o) * wrow + (uint32_t)j0);
                uint32_t wv[VEC];
                if constexpr (VEC == 1) {
                    wv[0] = wp[0];
                } else if constexpr (VEC == 2) {
                    const uint2 t = *reinterpret_cast<const uint2*>(wp);
                    wv[0] = t.x; wv[1] = t.y;
                } else {
                    const uint4 t = *reinterpret_cast<const uint4*>(wp);
                    wv[0] = t.x; wv[1] = t.y; wv[2] = t.z; wv[3] = t.w;
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < VEC; ++j)
                        acc[i][o] += __builtin_popcount(xv[i][j] ^ wv[j]);
            }
        }

        // fold this branch into the float sums: y_t = c_in - 2*popcount
        const float* gp = scale + (size_t)tap * s.c_out + (FULL ? o0 : 0);
#pragma unroll
        for (int o = 0; o < TN; ++o) {
            float g;
            if constexpr (FULL) g = gp[o];
            else g = scale[(uint32_t)(tap * s.c_out) + chan(o)];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const float y = (float)(c_in - 2 * acc[i][o]);
                const float zn = __builtin_fmaf(g, y, z[i][o]);
                if constexpr (PADMODE == PAD_SKIP) z[i][o] = inb[i] ? zn : z[i][o];
                else z[i][o] = zn;
            }
        }
    }

    if constexpr (WAVE_EPILOGUE) {
        uint32_t* my_tile = ep_tile + wave * (64 * valu::TROW);
        const valu::Tile<true> t = valu::Tile<true>::make(ctile, s.c_out);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m_first = mtile * (64 * TM) + i * 64;
            if constexpr (OUT == OUT_F32)
                valu::store_words_wave(s, t, m_first, lane, false, z[i], static_cast<uint32_t*>(out), my_tile);
            else
                valu::module_store_wave<OUT == OUT_TAIL_F16, false>(s, ep, t, m_first, ctile, lane, z[i], my_tile);
        }
    } else if constexpr (FUSED) {
        uint32_t* zp = static_cast<uint32_t*>(out);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint32_t word = 0;
#pragma unroll
            for (int o = 0; o < TN; ++o) {
                const bool on = (FULL || o0 + o <= o_last) && (z[i][o] >= 0.0f);
                word |= (uint32_t)on << o;
            }
            if (live[i]) {
                const int m = mtile * (64 * TM) + i * 64 + lane;
                zp[(size_t)m * s.cwo + ctile] = word >> shift;
            }
        }
    } else {
        float* zo = static_cast<float*>(out);
        const bool vec_ok = FULL && (s.c_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(zo) & 15) == 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (!live[i]) continue;
            const int m = mtile * (64 * TM) + i * 64 + lane;
            float* row = zo + (size_t)m * s.c_out + o0;
            if (vec_ok) {
#pragma unroll
                for (int o = 0; o < TN; o += 4)
                    if (o >= shift)
                        *reinterpret_cast<float4*>(row + o) =
                            make_float4(z[i][o], z[i][o + 1], z[i][o + 2], z[i][o + 3]);
            } else {
#pragma unroll
                for (int o = 0; o < TN; ++o)
                    if (o >= shift && o0 + o < s.c_out) row[o] = z[i][o];
            }
        }
    }
}

template <int TM, int VEC, int PADMODE>
hipError_t launch_mode(const ConvShape& s, const BranchArgs& a, hipStream_t stream)
{
    const int n_ctiles = (s.c_out + TN - 1) / TN;
    const int n_mtiles = (s.m + 64 * TM - 1) / (64 * TM);
    const int64_t waves = (int64_t)n_ctiles * n_mtiles;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    const ModuleEp ep = a.tail ? *a.tail : ModuleEp{};
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, stream, s, a.branches, n_mtiles, n_ctiles, a.x,
                           a.x_branch_stride, a.w, a.pad_words, a.scale, a.bias, a.out, ep);
    };
    const bool full = s.c_out >= TN;
    if (a.tail) {
        if (!full) return hipErrorInvalidValue;     // the caller routes c_out < 32 elsewhere
        if (ep.half) go(conv_branches_kernel<TM, VEC, PADMODE, OUT_TAIL_F16, true>);
        else go(conv_branches_kernel<TM, VEC, PADMODE, OUT_TAIL_F32, true>);
    } else if (a.fused) {
        if (full) go(conv_branches_kernel<TM, VEC, PADMODE, OUT_BITS, true>);
        else go(conv_branches_kernel<TM, VEC, PADMODE, OUT_BITS, false>);
    } else {
        if (full) go(conv_branches_kernel<TM, VEC, PADMODE, OUT_F32, true>);
        else go(conv_branches_kernel<TM, VEC, PADMODE, OUT_F32, false>);
    }
    return hipGetLastError();
}

template <int TM, int VEC>
hipError_t launch_vec(const ConvShape& s, const BranchArgs& a, hipStream_t stream)
{
    if (a.zero_pad) return launch_mode<TM, VEC, PAD_SKIP>(s, a, stream);
    if (a.pad_words) return launch_mode<TM, VEC, PAD_WORDS>(s, a, stream);
    return launch_mode<TM, VEC, PAD_MINUS>(s, a, stream);
}

template <int TM>
hipError_t launch_tm(const ConvShape& s, const BranchArgs& a, hipStream_t stream)
{
    // every vector load must be aligned: tensors, the distance between the
    // branches' tensors, and the words per pixel
    const uintptr_t bits = reinterpret_cast<uintptr_t>(a.x) | reinterpret_cast<uintptr_t>(a.w) |
                           ((uintptr_t)a.x_branch_stride * 4u);
    if (s.cw % 4 == 0 && (bits & 15) == 0) return launch_vec<TM, 4>(s, a, stream);
    if (s.cw % 2 == 0 && (bits & 7) == 0) return launch_vec<TM, 2>(s, a, stream);
    return launch_vec<TM, 1>(s, a, stream);
}

}  // namespace

hipError_t launch_conv_branches(const ConvShape& s, const BranchArgs& a, hipStream_t stream)
{
    // two pixels per lane unless one pixel per lane spreads a launch of a few
    // workgroups per compute unit better (same rule as the plain vector-ALU kernel)
    const int64_t n_ct = (s.c_out + TN - 1) / TN;
    const int64_t waves2 = n_ct * ((s.m + 127) / 128), waves1 = n_ct * ((s.m + 63) / 64);
    const int64_t rounds2 = ((waves2 + 3) / 4 + 255) / 256, rounds1 = ((waves1 + 3) / 4 + 255) / 256;
    if (waves2 >= 2048 && 20 * rounds2 <= 11 * rounds1) return launch_tm<2>(s, a, stream);
    return launch_tm<1>(s, a, stream);
}

}  // namespace bcnn
