// Binary convolution on the vector ALUs: implicit GEMM over packed words,
//   dot = K - 2 * sum_words popcount(x_word xor w_word)
// (BCNN paper, Section 1: the operator lowers to a matrix product; Section
// 4.2.1: operands are +-1).  No im2col buffer exists anywhere.
//
// Mapping.  A wave owns 64*TM output pixels (one or more per lane) and TN = 32
// consecutive output channels, i.e. exactly one packed output word per pixel.
// The weights of a wave are the same for all of its lanes, so they are read
// with scalar loads into SGPRs and enter v_xor_b32 as the scalar operand:
// weights cost no vector-memory or LDS bandwidth and no VGPRs.  Each lane
// loads its own pixels' packed input words (VEC words at a time) straight from
// global memory; a tap outside the image is the all-zero word (-1 in every
// channel), so borders need no correction term.  Per VEC input words a lane
// issues VEC*TM*TN xor+popcount pairs, so vector loads are <1% of the
// instruction stream and latency is hidden by the other waves of the SIMD.
//
// Channel tiles.  With c_out >= 32 (FULL) every tile computes 32 real channels:
// the last tile of a ragged c_out starts at c_out - 32 instead of 32*ctile and
// drops the `shift` channels it shares with its neighbour when it stores, so no
// index is ever clamped and per-channel parameters are plain contiguous scalar
// loads.  With c_out < 32 rows beyond c_out are clamped to the last real one so
// that every scalar load stays inside its tensor.
#include "valu_epilogue.h"

namespace bcnn {
namespace {

using valu::TN;
using valu::Tile;

enum { OUT_I32 = 0, OUT_BITS = 1, OUT_MODULE_F32 = 2, OUT_MODULE_F16 = 3, OUT_MODULE_BF16 = 4 };   // module: 2 + REAL_*

template <int VEC>
__device__ __forceinline__ void load_words(const uint32_t* p, bool ok, uint32_t (&out)[VEC])
{
    if constexpr (VEC == 1) {
        out[0] = ok ? *p : 0u;
    } else if constexpr (VEC == 2) {
        uint2 v = ok ? *reinterpret_cast<const uint2*>(p) : make_uint2(0u, 0u);
        out[0] = v.x; out[1] = v.y;
    } else {
        uint4 v = ok ? *reinterpret_cast<const uint4*>(p) : make_uint4(0u, 0u, 0u, 0u);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
}

template <int TM, int VEC, int OUT, bool FULL>
__global__ __launch_bounds__(256) void conv_valu_kernel(
    ConvShape s, int32_t n_mtiles, int32_t n_ctiles,
    const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out, ModuleEp ep)
{
    // full tiles with 32-bit or real outputs leave through a per-wave LDS tile (valu_epilogue.h)
    constexpr bool WAVE_EPILOGUE = FULL && OUT != OUT_BITS;
    __shared__ uint32_t ep_tile[WAVE_EPILOGUE ? 4 * 64 * valu::TROW : 1];
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int tile = blockIdx.x * 4 + wave;
    // channel tile fastest: the waves that share one pixel tile run together
    const int ctile = tile % n_ctiles;
    const int mtile = tile / n_ctiles;
    if (mtile >= n_mtiles) return;
    const Tile<FULL> t = Tile<FULL>::make(ctile, s.c_out);

    // 1x1 with unit stride: output pixel m reads input pixel m, no coordinates needed
    const bool direct = s.ks == 1 && s.stride == 1;
    int pn[TM], ph[TM], pw[TM], pm[TM];
    bool live[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = mtile * (64 * TM) + i * 64 + lane;
        live[i] = m < s.m;
        const int mc = live[i] ? m : s.m - 1;
        pm[i] = mc;
        pn[i] = ph[i] = pw[i] = 0;
        if (!direct) {
            const int hw = s.ho * s.wo;
            pn[i] = mc / hw;
            const int r = mc - pn[i] * hw;
            const int oh = r / s.wo;
            ph[i] = oh * s.stride - s.pad;
            pw[i] = (r - oh * s.wo) * s.stride - s.pad;
        }
    }

    int32_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int o = 0; o < TN; ++o) acc[i][o] = 0;

    const int taps = s.ks * s.ks;
    const uint32_t wrow = (uint32_t)(taps * s.cw);  // words per output channel

    for (int tap = 0; tap < taps; ++tap) {
        const int u = tap / s.ks, v = tap - u * s.ks;
        const uint32_t* xp[TM];
        bool inb[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (direct) {
                inb[i] = true;
                xp[i] = x + (size_t)pm[i] * s.cw;
            } else {
                const int ih = ph[i] + u, iw = pw[i] + v;
                inb[i] = ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
                const int ihc = inb[i] ? ih : 0, iwc = inb[i] ? iw : 0;
                xp[i] = x + ((size_t)(pn[i] * s.h + ihc) * s.w + iwc) * s.cw;
            }
        }
        const uint32_t* wt = w + (uint32_t)(tap * s.cw);
        for (int j0 = 0; j0 < s.cw; j0 += VEC) {
            uint32_t xv[TM][VEC];
#pragma unroll
            for (int i = 0; i < TM; ++i) load_words<VEC>(xp[i] + j0, inb[i], xv[i]);
#pragma unroll
            for (int o = 0; o < TN; ++o) {
                const uint32_t* wp = wt + (t.chan(o) * wrow + (uint32_t)j0);
                uint32_t wv[VEC];
                if constexpr (VEC == 1) {
                    wv[0] = wp[0];
                } else if constexpr (VEC == 2) {
                    const uint2 q = *reinterpret_cast<const uint2*>(wp);
                    wv[0] = q.x; wv[1] = q.y;
                } else {
                    const uint4 q = *reinterpret_cast<const uint4*>(wp);
                    wv[0] = q.x; wv[1] = q.y; wv[2] = q.z; wv[3] = q.w;
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < VEC; ++j)
                        acc[i][o] += __builtin_popcount(xv[i][j] ^ wv[j]);
            }
        }
    }

    // Epilogue.  dot = K - 2*popcount; padding needs no correction because
    // padded taps were real all-zero words.
    if constexpr (WAVE_EPILOGUE) {
        uint32_t* my_tile = ep_tile + wave * (64 * valu::TROW);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m_first = mtile * (64 * TM) + i * 64;
            if constexpr (OUT == OUT_I32)
                valu::store_words_wave(s, t, m_first, lane, true, acc[i], static_cast<uint32_t*>(out), my_tile);
            else
                valu::module_store_wave<OUT - OUT_MODULE_F32, true>(s, ep, t, m_first, ctile, lane, acc[i], my_tile);
        }
    } else if constexpr (OUT >= OUT_MODULE_F32) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            if (live[i])
                valu::module_store<OUT - OUT_MODULE_F32, FULL, true>(s, ep, t, mtile * (64 * TM) + i * 64 + lane,
                                                                      ctile, acc[i]);
    } else if constexpr (OUT == OUT_BITS) {
        uint32_t* yp = static_cast<uint32_t*>(out);
        const int32_t* tp = thr + (FULL ? t.o0 : 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint32_t word = 0;
#pragma unroll
            for (int o = 0; o < TN; ++o) {
                int32_t th;
                if constexpr (FULL) th = tp[o];
                else th = tp[t.chan(o)];
                const bool on = (FULL || t.stores(o)) && (s.k - 2 * acc[i][o] >= th);
                word |= (uint32_t)on << o;
            }
            if (live[i]) {
                const int m = mtile * (64 * TM) + i * 64 + lane;
                yp[(size_t)m * s.cwo + ctile] = word >> t.shift;
            }
        }
    } else {
        int32_t* y = static_cast<int32_t*>(out);
        const bool vec_ok = FULL && (s.c_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) & 15) == 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (!live[i]) continue;
            const int m = mtile * (64 * TM) + i * 64 + lane;
            int32_t* row = y + (size_t)m * s.c_out + t.o0;
            if (vec_ok) {
#pragma unroll
                for (int o = 0; o < TN; o += 4) {
                    int4 q;
                    q.x = s.k - 2 * acc[i][o + 0];
                    q.y = s.k - 2 * acc[i][o + 1];
                    q.z = s.k - 2 * acc[i][o + 2];
                    q.w = s.k - 2 * acc[i][o + 3];
                    if (o >= t.shift) *reinterpret_cast<int4*>(row + o) = q;
                }
            } else {
#pragma unroll
                for (int o = 0; o < TN; ++o)
                    if (t.stores(o)) row[o] = s.k - 2 * acc[i][o];
            }
        }
    }
}

// ---- tiny problems ---------------------------------------------------------
// With a handful of waves in the whole launch nothing hides the latency of the
// main kernel's chain of scalar weight loads (32 channels x taps, one after the
// other).  Here a wave (one per block, 64 pixels x 32 channels as above) fetches
// everything it needs up front with vector loads, so it pays one memory latency:
// its pixels' input words (one register per word) and its 32 weight rows
// (register r: word 2r of channel `lane` in lanes 0-31, word 2r+1 in lanes 32-63).
// v_readlane then turns a weight word into the scalar operand of v_xor_b32.
// Covers taps * cw <= 2 * SMALL_REGS words per weight row.
constexpr int SMALL_REGS = 18;

template <int OUT, bool FULL>
__global__ __launch_bounds__(64) void conv_valu_small_kernel(
    ConvShape s, int32_t n_ctiles, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out)
{
    const int lane = threadIdx.x;
    const int ctile = blockIdx.x % n_ctiles;
    const int mtile = blockIdx.x / n_ctiles;
    const Tile<FULL> t = Tile<FULL>::make(ctile, s.c_out);

    const int m = mtile * 64 + lane;
    const bool live = m < s.m;
    const int mc = live ? m : s.m - 1;
    const int hw = s.ho * s.wo;
    const int pn = mc / hw;
    const int rr = mc - pn * hw;
    const int oh = rr / s.wo;
    const int ph = oh * s.stride - s.pad;
    const int pw = (rr - oh * s.wo) * s.stride - s.pad;

    const int row_words = s.ks * s.ks * s.cw;     // words per weight row = per pixel window
    // weights: lane's channel (lanes 32-63 take the same channels again, odd words)
    const uint32_t* wrow = w + (size_t)t.chan(lane & 31) * row_words + (lane >> 5);
    uint32_t wr[SMALL_REGS];
#pragma unroll
    for (int r = 0; r < SMALL_REGS; ++r) {
        const int word = 2 * r + (lane >> 5);
        wr[r] = word < row_words ? wrow[2 * r] : 0u;
    }
    // inputs: word k of the lane's window = tap k / cw, channel word k % cw
    uint32_t xr[2 * SMALL_REGS];
    {
        int j = 0, u = 0, v = 0;                 // channel word, filter row, filter column of word k
#pragma unroll
        for (int k = 0; k < 2 * SMALL_REGS; ++k) {
            const int ih = ph + u, iw = pw + v;
            const bool ok = k < row_words && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            xr[k] = ok ? x[((size_t)(pn * s.h + ih) * s.w + iw) * s.cw + j] : 0u;
            if (++j == s.cw) {
                j = 0;
                if (++v == s.ks) { v = 0; ++u; }
            }
        }
    }

    int32_t acc[TN];
#pragma unroll
    for (int o = 0; o < TN; ++o) acc[o] = 0;
#pragma unroll
    for (int r = 0; r < SMALL_REGS; ++r) {
        if (2 * r < row_words) {
#pragma unroll
            for (int o = 0; o < TN; ++o)
                acc[o] += __builtin_popcount(xr[2 * r] ^ (uint32_t)__builtin_amdgcn_readlane((int)wr[r], o));
        }
        if (2 * r + 1 < row_words) {
#pragma unroll
            for (int o = 0; o < TN; ++o)
                acc[o] += __builtin_popcount(xr[2 * r + 1] ^ (uint32_t)__builtin_amdgcn_readlane((int)wr[r], 32 + o));
        }
    }

    if constexpr (OUT == OUT_BITS) {
        uint32_t word = 0;
#pragma unroll
        for (int o = 0; o < TN; ++o) {
            const bool on = (FULL || t.stores(o)) && (s.k - 2 * acc[o] >= thr[t.chan(o)]);
            word |= (uint32_t)on << o;
        }
        if (live) static_cast<uint32_t*>(out)[(size_t)m * s.cwo + ctile] = word >> t.shift;
    } else {
        if (live) {
            int32_t* row = static_cast<int32_t*>(out) + (size_t)m * s.c_out + t.o0;
#pragma unroll
            for (int o = 0; o < TN; ++o)
                if (t.stores(o)) row[o] = s.k - 2 * acc[o];
        }
    }
}

// The same for int32 sums with only CT output channels per wave: the sums need
// no packing, so the channels can be spread over eight times as many waves, each
// with an eighth of the instruction chain (a tiny problem is nothing but that
// chain: 64 waves of 430 instructions instead of 8 of 3500).
template <int CT>
__global__ __launch_bounds__(64) void conv_valu_small_split_kernel(
    ConvShape s, int32_t n_ctiles, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    int32_t* __restrict__ y)
{
    static_assert(CT <= 32, "a lane half holds one channel per lane");
    const int lane = threadIdx.x;
    const int ctile = blockIdx.x % n_ctiles;
    const int mtile = blockIdx.x / n_ctiles;
    const int o0 = ctile * CT;

    const int m = mtile * 64 + lane;
    const bool live = m < s.m;
    const int mc = live ? m : s.m - 1;
    const int hw = s.ho * s.wo;
    const int pn = mc / hw;
    const int rr = mc - pn * hw;
    const int oh = rr / s.wo;
    const int ph = oh * s.stride - s.pad;
    const int pw = (rr - oh * s.wo) * s.stride - s.pad;

    const int row_words = s.ks * s.ks * s.cw;
    // weights: lane l < 32 holds even words of channel o0 + l % CT, lane 32 + l the odd ones
    int wch = o0 + (lane & 31) % CT;
    wch = wch < s.c_out ? wch : s.c_out - 1;
    const uint32_t* wrow = w + (size_t)wch * row_words + (lane >> 5);
    uint32_t wr[SMALL_REGS];
#pragma unroll
    for (int r = 0; r < SMALL_REGS; ++r) {
        const int word = 2 * r + (lane >> 5);
        wr[r] = word < row_words ? wrow[2 * r] : 0u;
    }
    uint32_t xr[2 * SMALL_REGS];
    {
        int j = 0, u = 0, v = 0;                 // channel word, filter row, filter column of word k
#pragma unroll
        for (int k = 0; k < 2 * SMALL_REGS; ++k) {
            const int ih = ph + u, iw = pw + v;
            const bool ok = k < row_words && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            xr[k] = ok ? x[((size_t)(pn * s.h + ih) * s.w + iw) * s.cw + j] : 0u;
            if (++j == s.cw) {
                j = 0;
                if (++v == s.ks) { v = 0; ++u; }
            }
        }
    }
    int32_t acc[CT];
#pragma unroll
    for (int o = 0; o < CT; ++o) acc[o] = 0;
#pragma unroll
    for (int r = 0; r < SMALL_REGS; ++r) {
        if (2 * r < row_words) {
#pragma unroll
            for (int o = 0; o < CT; ++o)
                acc[o] += __builtin_popcount(xr[2 * r] ^ (uint32_t)__builtin_amdgcn_readlane((int)wr[r], o));
        }
        if (2 * r + 1 < row_words) {
#pragma unroll
            for (int o = 0; o < CT; ++o)
                acc[o] += __builtin_popcount(xr[2 * r + 1] ^ (uint32_t)__builtin_amdgcn_readlane((int)wr[r], 32 + o));
        }
    }
    if (live) {
        int32_t* row = y + (size_t)m * s.c_out + o0;
#pragma unroll
        for (int o = 0; o < CT; ++o)
            if (o0 + o < s.c_out) row[o] = s.k - 2 * acc[o];
    }
}

// ---- few waves, long weight rows ---------------------------------------------
// Between the tiny problems above and the launches that fill the chip several
// times over lies a gap: some tens to a couple of thousand waves, weight rows
// longer than the tiny kernel's 36 words.  The main kernel is latency bound
// there (nothing hides its scalar weight loads: 3x3, 192 -> 64 channels on 1568
// pixels took 35 us where the instructions alone need 7).  This kernel keeps the
// tiny kernel's way of getting weights (vector loads, v_readlane to broadcast)
// and walks the weight row in chunks of 16 words, the next chunk's weights and
// inputs being fetched while the current one is multiplied.  Three instructions
// per word and channel instead of two, so it only serves launches that cannot
// fill the chip.
constexpr int CHUNK_WORDS = 16;

template <int OUT, bool FULL>
__global__ __launch_bounds__(64) void conv_valu_chunked_kernel(
    ConvShape s, int32_t n_ctiles, const uint32_t* __restrict__ x, const uint32_t* __restrict__ w,
    const int32_t* __restrict__ thr, void* __restrict__ out)
{
    constexpr int WR = CHUNK_WORDS / 2;           // weight registers per chunk: lane half h holds words 8h .. 8h+7
    const int lane = threadIdx.x;
    const int half = lane >> 5;
    const int ctile = blockIdx.x % n_ctiles;
    const int mtile = blockIdx.x / n_ctiles;
    const Tile<FULL> t = Tile<FULL>::make(ctile, s.c_out);

    const int m = mtile * 64 + lane;
    const bool live = m < s.m;
    const int mc = live ? m : s.m - 1;
    const int hw = s.ho * s.wo;
    const int pn = mc / hw;
    const int rr = mc - pn * hw;
    const int oh = rr / s.wo;
    const int ph = oh * s.stride - s.pad;
    const int pw = (rr - oh * s.wo) * s.stride - s.pad;

    const int row_words = s.ks * s.ks * s.cw;
    const int n_chunks = (row_words + CHUNK_WORDS - 1) / CHUNK_WORDS;
    const uint32_t* wrow = w + (size_t)t.chan(lane & 31) * row_words + WR * half;

    // position (channel word j, filter row u, filter column v) of the next input word to fetch
    int fj = 0, fu = 0, fv = 0, fk = 0;
    auto fetch = [&](uint32_t (&wr)[WR], uint32_t (&xr)[CHUNK_WORDS], int chunk) {
#pragma unroll
        for (int r = 0; r < WR; ++r) {
            const int word = chunk * CHUNK_WORDS + WR * half + r;
            wr[r] = word < row_words ? wrow[chunk * CHUNK_WORDS + r] : 0u;
        }
#pragma unroll
        for (int r = 0; r < CHUNK_WORDS; ++r) {
            const int ih = ph + fu, iw = pw + fv;
            const bool ok = fk < row_words && ih >= 0 && ih < s.h && iw >= 0 && iw < s.w;
            xr[r] = ok ? x[((size_t)(pn * s.h + ih) * s.w + iw) * s.cw + fj] : 0u;
            ++fk;
            if (++fj == s.cw) {
                fj = 0;
                if (++fv == s.ks) { fv = 0; ++fu; }
            }
        }
    };

    int32_t acc[TN];
#pragma unroll
    for (int o = 0; o < TN; ++o) acc[o] = 0;
    uint32_t wc[WR], xc[CHUNK_WORDS], wn[WR], xn[CHUNK_WORDS];
    fetch(wc, xc, 0);
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        if (chunk + 1 < n_chunks) {
            fetch(wn, xn, chunk + 1);
        } else {
#pragma unroll
            for (int r = 0; r < WR; ++r) wn[r] = 0u;
#pragma unroll
            for (int r = 0; r < CHUNK_WORDS; ++r) xn[r] = 0u;
        }
        // words past the end of the row are zero on both sides and count nothing
#pragma unroll
        for (int r = 0; r < CHUNK_WORDS; ++r)
#pragma unroll
            for (int o = 0; o < TN; ++o)
                acc[o] += __builtin_popcount(
                    xc[r] ^ (uint32_t)__builtin_amdgcn_readlane((int)wc[r % WR], 32 * (r / WR) + o));
#pragma unroll
        for (int r = 0; r < WR; ++r) wc[r] = wn[r];
#pragma unroll
        for (int r = 0; r < CHUNK_WORDS; ++r) xc[r] = xn[r];
    }

    if constexpr (OUT == OUT_BITS) {
        uint32_t word = 0;
#pragma unroll
        for (int o = 0; o < TN; ++o) {
            const bool on = (FULL || t.stores(o)) && (s.k - 2 * acc[o] >= thr[t.chan(o)]);
            word |= (uint32_t)on << o;
        }
        if (live) static_cast<uint32_t*>(out)[(size_t)m * s.cwo + ctile] = word >> t.shift;
    } else {
        if (live) {
            int32_t* row = static_cast<int32_t*>(out) + (size_t)m * s.c_out + t.o0;
#pragma unroll
            for (int o = 0; o < TN; ++o)
                if (t.stores(o)) row[o] = s.k - 2 * acc[o];
        }
    }
}

bool chunked_applies(const ConvShape& s)
{
    const int64_t waves = (int64_t)((s.c_out + TN - 1) / TN) * ((s.m + 63) / 64);
    return s.ks * s.ks * s.cw >= 24 && waves <= 2048;
}

hipError_t launch_chunked(const ConvShape& s, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                          void* out, hipStream_t stream)
{
    const int n_ctiles = (s.c_out + TN - 1) / TN;
    const unsigned blocks = (unsigned)(n_ctiles * ((s.m + 63) / 64));
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(64), 0, stream, s, n_ctiles, x, w, thr, out);
    };
    const bool full = s.c_out >= TN;
    if (thr) {
        if (full) go(conv_valu_chunked_kernel<OUT_BITS, true>);
        else go(conv_valu_chunked_kernel<OUT_BITS, false>);
    } else {
        if (full) go(conv_valu_chunked_kernel<OUT_I32, true>);
        else go(conv_valu_chunked_kernel<OUT_I32, false>);
    }
    return hipGetLastError();
}

// Whether the tiny-problem kernel applies, and its launch.
bool small_applies(const ConvShape& s)
{
    const int64_t waves = (int64_t)((s.c_out + TN - 1) / TN) * ((s.m + 63) / 64);
    return s.ks * s.ks * s.cw <= 2 * SMALL_REGS && waves <= 256;
}

hipError_t launch_small(const ConvShape& s, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                        void* out, hipStream_t stream)
{
    const int n_ctiles = (s.c_out + TN - 1) / TN;
    const unsigned blocks = (unsigned)(n_ctiles * ((s.m + 63) / 64));
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(64), 0, stream, s, n_ctiles, x, w, thr, out);
    };
    if (!thr) {        // int32 sums: four channels per wave
        constexpr int CT = 4;
        const int split_ctiles = (s.c_out + CT - 1) / CT;
        hipLaunchKernelGGL((conv_valu_small_split_kernel<CT>), dim3((unsigned)(split_ctiles * ((s.m + 63) / 64))),
                           dim3(64), 0, stream, s, split_ctiles, x, w, static_cast<int32_t*>(out));
        return hipGetLastError();
    }
    if (s.c_out >= TN) go(conv_valu_small_kernel<OUT_BITS, true>);
    else go(conv_valu_small_kernel<OUT_BITS, false>);
    return hipGetLastError();
}

template <int TM, int VEC, int OUT>
hipError_t launch_out(const ConvShape& s, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                      void* out, const ModuleEp& ep, hipStream_t stream)
{
    const int n_ctiles = (s.c_out + TN - 1) / TN;
    const int n_mtiles = (s.m + 64 * TM - 1) / (64 * TM);
    const int64_t waves = (int64_t)n_ctiles * n_mtiles;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    if (s.c_out >= TN)
        hipLaunchKernelGGL((conv_valu_kernel<TM, VEC, OUT, true>), dim3(blocks), dim3(256), 0, stream,
                           s, n_mtiles, n_ctiles, x, w, thr, out, ep);
    else
        hipLaunchKernelGGL((conv_valu_kernel<TM, VEC, OUT, false>), dim3(blocks), dim3(256), 0, stream,
                           s, n_mtiles, n_ctiles, x, w, thr, out, ep);
    return hipGetLastError();
}

template <int TM, int VEC>
hipError_t launch_tm_vec(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                         const int32_t* thr, void* out, const ModuleEp* ep, hipStream_t stream)
{
    const ModuleEp none = {};
    if (ep && ep->half == REAL_BF16) return launch_out<TM, VEC, OUT_MODULE_BF16>(s, x, w, thr, out, *ep, stream);
    if (ep && ep->half) return launch_out<TM, VEC, OUT_MODULE_F16>(s, x, w, thr, out, *ep, stream);
    if (ep) return launch_out<TM, VEC, OUT_MODULE_F32>(s, x, w, thr, out, *ep, stream);
    if (thr) return launch_out<TM, VEC, OUT_BITS>(s, x, w, thr, out, none, stream);
    return launch_out<TM, VEC, OUT_I32>(s, x, w, thr, out, none, stream);
}

template <int TM>
hipError_t launch_tm(const ConvShape& s, const uint32_t* x, const uint32_t* w, const int32_t* thr,
                     void* out, const ModuleEp* ep, hipStream_t stream)
{
    const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w);
    if (s.cw % 4 == 0 && (bits & 15) == 0) return launch_tm_vec<TM, 4>(s, x, w, thr, out, ep, stream);
    if (s.cw % 2 == 0 && (bits & 7) == 0) return launch_tm_vec<TM, 2>(s, x, w, thr, out, ep, stream);
    return launch_tm_vec<TM, 1>(s, x, w, thr, out, ep, stream);
}

}  // namespace

hipError_t launch_conv_valu(const ConvShape& s, const uint32_t* x, const uint32_t* w,
                            const int32_t* thr, void* out, const ModuleEp* ep, hipStream_t stream)
{
    // Two pixels per lane halve the scalar weight traffic per popcount (one
    // pixel per lane costs about 10 % more per popcount, measured); one pixel
    // per lane gives twice as many waves, which small problems need to cover
    // 1024 SIMDs and which evens out a launch of a few workgroups per compute
    // unit: all of them are resident at once, so the unit with the most
    // workgroups sets the time (784 workgroups of two pixels per lane are 4 on
    // some of the 256 units and 3 on the rest; 1568 of one pixel are 7 and 6).
    if (!ep && small_applies(s)) return launch_small(s, x, w, thr, out, stream);
    if (!ep && chunked_applies(s)) return launch_chunked(s, x, w, thr, out, stream);
    const int64_t n_ct = (s.c_out + TN - 1) / TN;
    const int64_t waves2 = n_ct * ((s.m + 127) / 128), waves1 = n_ct * ((s.m + 63) / 64);
    const int64_t rounds2 = ((waves2 + 3) / 4 + 255) / 256, rounds1 = ((waves1 + 3) / 4 + 255) / 256;
    if (waves2 >= 2048 && 20 * rounds2 <= 11 * rounds1) return launch_tm<2>(s, x, w, thr, out, ep, stream);
    return launch_tm<1>(s, x, w, thr, out, ep, stream);
}

}  // namespace bcnn
