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
template <bool HALF, bool FULL, bool FROM_SUMS, typename V>
__device__ __forceinline__ void module_store(const ConvShape& s, const ModuleEp& ep, const Tile<FULL>& t,
                                             int m, int ctile, const V (&vals)[TN])
{
    using real_t = typename std::conditional<HALF, _Float16, float>::type;
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
            v[o] = module_value<HALF>((float)(s.k - 2 * vals[o]), (ep.scale + ob)[oc], (ep.bias + ob)[oc],
                                      ep.identity != nullptr, idv[o], ep.slope != nullptr, slope);
        else
            v[o] = module_tail<HALF>(vals[o], ep.identity != nullptr, idv[o], ep.slope != nullptr, slope);
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

}  // namespace valu
}  // namespace bcnn
