// Shared by the vector-ALU kernels (plain and branch convolution): where a
// wave's 32-channel tile lives, and the module epilogue of one pixel.
#pragma once

#include "bcnn_common.h"

#include <type_traits>

namespace bcnn {
namespace valu {

constexpr int TN = 32;   // output channels per wave = one packed output word per pixel

// Where a tile's channels live: channel of accumulator o, and whether the tile
// stores it.
template <bool FULL>
struct Tile {
    int o0, shift, o_last;
    // FULL: the last tile of a ragged c_out starts at c_out - 32 and drops `shift` channels when it stores
    __device__ __forceinline__ static Tile make(int ctile, int c_out)
    {
        Tile t;
        t.o_last = c_out - 1;
        t.o0 = (FULL && ctile * TN + TN > c_out) ? c_out - TN : ctile * TN;
        t.shift = ctile * TN - t.o0;
        return t;
    }
    __device__ __forceinline__ uint32_t chan(int o) const
    {
        if constexpr (FULL) return (uint32_t)(o0 + o);
        else return (uint32_t)((o0 + o < o_last) ? (o0 + o) : o_last);
    }
    __device__ __forceinline__ bool stores(int o) const
    {
        if constexpr (FULL) return o >= shift;
        else return o0 + o <= o_last;
    }
};

// Module epilogue for one pixel of a lane.  The lane's 32 values are contiguous
// in the real stream (128 or 64 bytes); when everything is 16-byte aligned
// they move as 16-byte vectors, all loads before any store (the stream may be
// updated in place).
//
// FROM_SUMS: `vals` are the popcounts of a plain convolution (y = K - 2*vals,
// batch-norm scale and bias applied here); otherwise they are the float sums
// of a branch convolution, which already carry their scales and bias.
template <int REAL, bool FULL, bool FROM_SUMS, typename V>
__device__ __forceinline__ void module_store(const ConvShape& s, const ModuleEp& ep, const Tile<FULL>& t,
                                             int m, int ctile, const V (&vals)[TN])
{
    constexpr bool HALF = REAL != REAL_F32;             // a 16-bit stream
    using real_t = typename real_type<REAL>::type;
    constexpr int PER = HALF ? 8 : 4;                  // elements per 16-byte vector
    typedef real_t realv __attribute__((ext_vector_type(PER)));
    const size_t row = (size_t)m * s.c_out + t.o0;
    // the identity stream may have fewer channels than the output (replication by
    // bookkeeping): channel o reads o mod id_channels
    const int idc = ep.id_channels;
    const int id0 = t.o0 % idc;
    const real_t* idrow = static_cast<const real_t*>(ep.identity) + (size_t)m * idc;
    const real_t* idp = idrow + id0;
    real_t* rp = static_cast<real_t*>(ep.r) + row;
    const bool vec = FULL && (s.c_out % PER == 0) && (idc % PER == 0) && (id0 + TN <= idc) &&
                     ((reinterpret_cast<uintptr_t>(ep.identity) | reinterpret_cast<uintptr_t>(ep.r)) & 15) == 0;
    float idv[TN];
#pragma unroll
    for (int o = 0; o < TN; ++o) idv[o] = 0.0f;
    if (ep.identity) {
        if (vec) {
#pragma unroll
            for (int q = 0; q < TN / PER; ++q) {
                const realv v = __builtin_nontemporal_load(reinterpret_cast<const realv*>(idp) + q);
#pragma unroll
                for (int k = 0; k < PER; ++k) idv[q * PER + k] = (float)v[k];
            }
        } else {
#pragma unroll
            for (int o = 0; o < TN; ++o)
                if (FULL || t.stores(o)) idv[o] = (float)idrow[(id0 + o) % idc];
        }
    }
    const int ob = FULL ? t.o0 : 0;                    // FULL: plain offsets from the tile's first channel
    float v[TN];
    uint32_t word = 0;
#pragma unroll
    for (int o = 0; o < TN; ++o) {
        const int oc = FULL ? o : (int)t.chan(o);
        const float slope = ep.slope ? (ep.slope + ob)[oc] : 1.0f;
        if constexpr (FROM_SUMS)
            v[o] = module_value<REAL>((float)(s.k - 2 * vals[o]), (ep.scale + ob)[oc], (ep.bias + ob)[oc],
                                      ep.identity != nullptr, idv[o], ep.slope != nullptr, slope);
        else
            v[o] = module_tail<REAL>(vals[o], ep.identity != nullptr, idv[o], ep.slope != nullptr, slope);
        const float c = ep.next_bias ? (ep.next_bias + ob)[oc] : 0.0f;
        word |= (uint32_t)((FULL || t.stores(o)) && (v[o] + c >= 0.0f)) << o;
    }
    if (ep.r) {
        if (vec) {
#pragma unroll
            for (int q = 0; q < TN / PER; ++q) {
                realv u;
#pragma unroll
                for (int k = 0; k < PER; ++k) u[k] = (real_t)v[q * PER + k];
                if (q * PER >= t.shift) reinterpret_cast<realv*>(rp)[q] = u;
            }
        } else {
#pragma unroll
            for (int o = 0; o < TN; ++o)
                if (t.stores(o)) rp[o] = (real_t)v[o];
        }
    }
    if (ep.x_next) ep.x_next[(size_t)m * s.cwo + ctile] = word >> t.shift;
}

// ---- the same for a whole wave on a full tile, transposed through LDS -------
// Written per lane, a store instruction touches 64 different cache lines with
// 16 bytes each.  Here the wave parks its 64 pixels x 32 values in LDS (row =
// lane = pixel), then lane l takes the four channels 4*(l%8).. of pixel
// 8k + l/8, k = 0..7: eight lanes cover the 128 (64) contiguous bytes of one
// pixel, an instruction moves eight whole pixels, and the packed word of a pixel
// is the OR of eight nibbles (three DPP steps).  Every lane of the wave must
// call these, live pixel or not.
constexpr int TROW = TN + 4;   // LDS row in words: rows stay 16-byte aligned, banks skewed by 4

template <typename V>
__device__ __forceinline__ void park_values(uint32_t* tile, int lane, int k_total, bool from_sums,
                                            const V (&vals)[TN])
{
#pragma unroll
    for (int q = 0; q < TN / 4; ++q) {
        uint4 u;
        if (from_sums) {
            u.x = (uint32_t)(k_total - 2 * (int)vals[4 * q + 0]);
            u.y = (uint32_t)(k_total - 2 * (int)vals[4 * q + 1]);
            u.z = (uint32_t)(k_total - 2 * (int)vals[4 * q + 2]);
            u.w = (uint32_t)(k_total - 2 * (int)vals[4 * q + 3]);
        } else {
            u.x = __float_as_uint((float)vals[4 * q + 0]);
            u.y = __float_as_uint((float)vals[4 * q + 1]);
            u.z = __float_as_uint((float)vals[4 * q + 2]);
            u.w = __float_as_uint((float)vals[4 * q + 3]);
        }
        *reinterpret_cast<uint4*>(tile + lane * TROW + 4 * q) = u;
    }
}

// Plain 32-bit outputs (int32 sums of a convolution, float sums of a branch
// convolution): out is [m][c_out] of 4-byte elements.
template <typename V>
__device__ __forceinline__ void store_words_wave(const ConvShape& s, const Tile<true>& t, int m_first, int lane,
                                                 bool from_sums, const V (&vals)[TN], uint32_t* out, uint32_t* tile)
{
    park_values(tile, lane, s.k, from_sums, vals);
    const int cg = lane & 7;
    const bool vec = (s.c_out % 4 == 0) && ((reinterpret_cast<uintptr_t>(out) & 15) == 0);
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int px = 8 * k + (lane >> 3);
        const int m = m_first + px;
        const uint4 q = *reinterpret_cast<const uint4*>(tile + px * TROW + 4 * cg);
        if (m < s.m) {
            uint32_t* dstp = out + (size_t)m * s.c_out + t.o0 + 4 * cg;
            if (vec) {
                if (4 * cg >= t.shift) __builtin_nontemporal_store(u4{q.x, q.y, q.z, q.w}, reinterpret_cast<u4*>(dstp));
            } else {
                if (4 * cg + 0 >= t.shift) dstp[0] = q.x;
                if (4 * cg + 1 >= t.shift) dstp[1] = q.y;
                if (4 * cg + 2 >= t.shift) dstp[2] = q.z;
                if (4 * cg + 3 >= t.shift) dstp[3] = q.w;
            }
        }
    }
}

// FAST: all 64 pixels exist, the tile is not a shifted last tile, rows are
// vector aligned and the module has every part (identity, real stream out,
// next bits): no per-element predicates, loads and stores issue back to back.
template <int REAL, bool FROM_SUMS, bool FAST>
__device__ __forceinline__ void module_store_wave_parked(const ConvShape& s, const ModuleEp& ep, const Tile<true>& t,
                                                         int m_first, int ctile, int lane, const uint32_t* tile)
{
    constexpr bool HALF = REAL != REAL_F32;             // a 16-bit stream
    using real_t = typename real_type<REAL>::type;
    typedef real_t real4 __attribute__((ext_vector_type(4)));
    const int cg = lane & 7;
    const int c0 = t.o0 + 4 * cg;                      // the lane's four channels (all real: full tile)
    float pg[4], pb[4], pa[4], pc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        pg[j] = FROM_SUMS ? ep.scale[c0 + j] : 1.0f;
        pb[j] = FROM_SUMS ? ep.bias[c0 + j] : 0.0f;
        pa[j] = ep.slope ? ep.slope[c0 + j] : 1.0f;
        pc[j] = ep.next_bias ? ep.next_bias[c0 + j] : 0.0f;
    }
    // the identity stream may have fewer channels than the output (replication by
    // bookkeeping): channel o reads o mod id_channels
    const int idc = ep.id_channels;
    const int id0 = c0 % idc;
    constexpr uintptr_t AL = HALF ? 7 : 15;
    const bool vec = FAST || ((s.c_out % 4 == 0) && (idc % 4 == 0) &&
                              ((reinterpret_cast<uintptr_t>(ep.identity) | reinterpret_cast<uintptr_t>(ep.r)) & AL) == 0);
    const bool has_id = FAST || ep.identity != nullptr;
    const bool has_slope = FAST || ep.slope != nullptr;    // a missing slope is the slope 1 (pa = 1: 1 * t is t)
    // all identity vectors first: the stream may be updated in place
    real4 idv[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int m = m_first + 8 * k + (lane >> 3);
        real4 v4 = {(real_t)0, (real_t)0, (real_t)0, (real_t)0};
        if constexpr (FAST) {
            v4 = __builtin_nontemporal_load(reinterpret_cast<const real4*>(
                static_cast<const real_t*>(ep.identity) + (size_t)m * idc + id0));
        } else if (ep.identity && m < s.m) {
            const real_t* idrow = static_cast<const real_t*>(ep.identity) + (size_t)m * idc;
            if (vec) {
                v4 = __builtin_nontemporal_load(reinterpret_cast<const real4*>(idrow + id0));
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) v4[j] = idrow[(id0 + j) % idc];
            }
        }
        idv[k] = v4;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int px = 8 * k + (lane >> 3);
        const int m = m_first + px;
        const uint4 q = *reinterpret_cast<const uint4*>(tile + px * TROW + 4 * cg);
        const uint32_t qv[4] = {q.x, q.y, q.z, q.w};
        float v[4];
        uint32_t nib = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (FROM_SUMS)
                v[j] = module_value<REAL>((float)(int)qv[j], pg[j], pb[j], has_id, (float)idv[k][j], has_slope, pa[j]);
            else
                v[j] = module_tail<REAL>(__uint_as_float(qv[j]), has_id, (float)idv[k][j], has_slope, pa[j]);
            nib |= (uint32_t)(v[j] + pc[j] >= 0.0f) << j;
        }
        if (FAST || (ep.r && m < s.m)) {
            real_t* rp = static_cast<real_t*>(ep.r) + (size_t)m * s.c_out + c0;
            if (vec) {
                real4 u;
#pragma unroll
                for (int j = 0; j < 4; ++j) u[j] = (real_t)v[j];
                if (FAST || 4 * cg >= t.shift) *reinterpret_cast<real4*>(rp) = u;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (4 * cg + j >= t.shift) rp[j] = (real_t)v[j];
            }
        }
        // the eight lanes of a pixel hold the 32 channels of its packed word
        uint32_t wd = nib << (4 * cg);
        wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
        wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
        wd |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)wd, 0x141, 0xF, 0xF, true);  // row_half_mirror
        if constexpr (FAST) {
            if (cg == 0) ep.x_next[(size_t)m * s.cwo + ctile] = wd;
        } else {
            if (ep.x_next && cg == 0 && m < s.m) ep.x_next[(size_t)m * s.cwo + ctile] = wd >> t.shift;
        }
    }
}

template <int REAL, bool FROM_SUMS, typename V>
__device__ __forceinline__ void module_store_wave(const ConvShape& s, const ModuleEp& ep, const Tile<true>& t,
                                                  int m_first, int ctile, int lane, const V (&vals)[TN],
                                                  uint32_t* tile)
{
    park_values(tile, lane, s.k, FROM_SUMS, vals);
    constexpr uintptr_t AL = REAL != REAL_F32 ? 7 : 15;
    const bool fast = ep.identity && ep.r && ep.x_next && t.shift == 0 && m_first + 64 <= s.m &&
                      s.c_out % 4 == 0 && ep.id_channels % 4 == 0 &&
                      ((reinterpret_cast<uintptr_t>(ep.identity) | reinterpret_cast<uintptr_t>(ep.r)) & AL) == 0;
    if (fast) module_store_wave_parked<REAL, FROM_SUMS, true>(s, ep, t, m_first, ctile, lane, tile);
    else module_store_wave_parked<REAL, FROM_SUMS, false>(s, ep, t, m_first, ctile, lane, tile);
}

}  // namespace valu
}  // namespace bcnn
