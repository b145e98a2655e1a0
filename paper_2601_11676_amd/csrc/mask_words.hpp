// One token's mask held in registers, shared by the one-token kernels.
#pragma once
#include "common.hpp"

namespace halo {

// The token's mask as up to four 64-bit words held in scalar registers (one ballot per
// 64 groups); every wave builds them itself, so no LDS and no workgroup barrier sit
// between the launch and the first weight load.  The four byte loads are issued
// together (clamped index, not a branch) so they cost one memory latency.
struct MaskWords {
    unsigned long long w[4];
    int count;
};

__device__ __forceinline__ MaskWords load_mask_words(const uint8_t *__restrict__ mask, int G, int lane)
{
    MaskWords mw;
    mw.count = 0;
    uint8_t v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int g = k * kWave + lane;
        v[k] = mask[g < G ? g : 0];
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int g = k * kWave + lane;
        mw.w[k] = __ballot(g < G && v[k] != 0);
        mw.count += __popcll(mw.w[k]);
    }
    return mw;
}

// The union of T tokens' masks ([T][G] bytes) in the same form: a group is in it if any token
// keeps it.  All T*4 byte loads are issued together.  TMAX bounds T at compile time.
template <int TMAX>
__device__ __forceinline__ MaskWords load_union_words(const uint8_t *__restrict__ mask, int T, int G, int lane)
{
    uint8_t v[TMAX][4];
#pragma unroll
    for (int t = 0; t < TMAX; ++t)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int g = k * kWave + lane;
            v[t][k] = mask[(size_t)(t < T ? t : T - 1) * G + (g < G ? g : 0)];
        }
    MaskWords mw;
    mw.count = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int g = k * kWave + lane;
        uint8_t any = 0;
#pragma unroll
        for (int t = 0; t < TMAX; ++t) any |= v[t][k];
        mw.w[k] = __ballot(g < G && any != 0);
        mw.count += __popcll(mw.w[k]);
    }
    return mw;
}

// The groups of `mw` in ascending order, written by ONE wave to list[0 .. count-1] (LDS or global).
__device__ __forceinline__ void write_group_list(const MaskWords &mw, int lane, int *list)
{
    int base = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if ((mw.w[k] >> lane) & 1ull) list[base + __popcll(mw.w[k] & ((1ull << lane) - 1ull))] = k * kWave + lane;
        base += __popcll(mw.w[k]);
    }
}

// index of the u-th surviving group (u < count), wave-uniform
__device__ __forceinline__ int nth_group(const MaskWords &mw, int u, int lane)
{
    int base = 0, g = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = __popcll(mw.w[k]);
        if (u >= base && u < base + c) {
            const bool mine = (mw.w[k] >> lane) & 1ull;
            const int before = __popcll(mw.w[k] & ((1ull << lane) - 1ull));
            const unsigned long long sel = __ballot(mine && before == u - base);
            g = k * kWave + __builtin_ctzll(sel);
        }
        base += c;
    }
    return g;
}

}  // namespace halo
