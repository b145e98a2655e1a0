// Workgroup-level routine for the Pred step's second half (paper Sec. III-B.2 / III-B.3):
// [optionally the predictor's second layer] -> importance rank -> priority index -> device
// -> surviving set, for ONE token.  Shared by the stand-alone kernels (mask.hip) and by the
// decode kernels that carry the next block's prediction in spare workgroups (ffn_decode.hip).
//
// Ranking by counting: rank(g) = number of groups that come before g under (score
// descending, lower index first on equal scores, NaN after every number).  The G x G
// comparisons are spread over all threads of the workgroup (each thread takes one group and
// one slice of the opponents; slices are summed with LDS atomics), so the step costs a few
// hundred cycles instead of a serial sweep.  Survivor positions come from wave ballots.
#pragma once
#include "common.hpp"

namespace halo {

__device__ __forceinline__ bool ranks_before(float sh, int h, float sg, int g)
{
    const bool nh = sh != sh, ng = sg != sg;
    if (nh | ng) return (nh & ng) ? (h < g) : ng;
    return (sh > sg) | ((sh == sg) & (h < g));
}

struct MaskShared {
    __attribute__((aligned(16))) float score[1024];
    int pos[1024];
    unsigned long long bits[16];
    int8_t prio[1024];
    uint8_t drop[128];
    uint8_t keep[1024];
};

// NT = threads in the workgroup (multiple of 64, <= 1024); G <= 1024.
// FUSED: scores are computed here from h (float [r]) and Bt ([G][r]) and also written out;
// otherwise they are read from `scores`.  All pointers are for this token already.
template <int NT, typename WT, bool FUSED>
__device__ __forceinline__ void mask_scores_block(
    MaskShared &sh, int tid, const float *__restrict__ h, const WT *__restrict__ Bt, int r,
    float *__restrict__ scores, int G, int K, const int8_t *__restrict__ prio_dev, int n_dev,
    const uint8_t *__restrict__ drop, int32_t *__restrict__ order, int8_t *__restrict__ group_dev,
    uint8_t *__restrict__ mask, int32_t *__restrict__ surv_idx, int32_t *__restrict__ n_surv)
{
    constexpr int kWaves = NT / kWave;
    constexpr int GB = NT >= 1024 ? 8 : 16;     // groups whose rows a wave fetches before reducing any
    const int wave = tid >> 6, lane = tid & 63;
    // Everything the head needs from memory -- schedule, loss outcomes, h, the first batch of
    // Bt rows -- is requested in one straight line (clamped addresses and selects, no branches),
    // so the workgroup pays one memory latency, not one per item.
    const void *anywhere = FUSED ? static_cast<const void *>(Bt) : static_cast<const void *>(scores);
    const int8_t *pp = K > 0 ? prio_dev + (tid < K ? tid : K - 1) : static_cast<const int8_t *>(anywhere);
    const uint8_t *dp = drop ? drop + (tid < n_dev ? tid : n_dev - 1) : static_cast<const uint8_t *>(anywhere);
    const int8_t pv = *pp;
    const uint8_t dv = *dp;
    const bool fast = FUSED && r <= 512;        // one 8-element piece of h and of every row per lane
    const bool on = lane * 8 < r;
    float hx[8];
    Piece8<WT> w[GB];
    auto load_batch = [&](int g0) {
#pragma unroll
        for (int b = 0; b < GB; ++b) {
            const int g = g0 + kWaves * b;
            const bool ok = on && g < G;
            w[b].load(Bt + (size_t)(g < G ? g : G - 1) * r + (on ? lane * 8 : 0));
            if (!ok) w[b].zero();
        }
    };
    if (fast) {
        load8(h + (on ? lane * 8 : 0), hx);
        if (!on) {
#pragma unroll
            for (int e = 0; e < 8; ++e) hx[e] = 0.0f;
        }
        load_batch(wave < G ? wave : 0);        // a wave beyond G loads (and later discards) batch 0
    }
    if (tid < K) sh.prio[tid] = pv;
    for (int p = tid + NT; p < K; p += NT) sh.prio[p] = prio_dev[p];
    if (tid < n_dev) sh.drop[tid] = drop ? dv : 0;
    for (int g = tid; g < 1024; g += NT) sh.pos[g] = 0;
    if (FUSED) {
        if (fast) {
            for (int g0 = wave; g0 < G; g0 += kWaves * GB) {
                if (g0 != wave) load_batch(g0);
                float p[GB];
#pragma unroll
                for (int b = 0; b < GB; ++b) {
                    p[b] = 0.0f;
                    float wf[8];
                    w[b].get(wf);
#pragma unroll
                    for (int e = 0; e < 8; ++e) p[b] = __builtin_fmaf(hx[e], wf[e], p[b]);
                }
                // the butterflies advance together, distance by distance
#define HALO_STEP(OFF)                                           \
    _Pragma("unroll") for (int b = 0; b < GB; ++b) p[b] = xor_add<OFF>(p[b]);
                HALO_STEP(32) HALO_STEP(16) HALO_STEP(8) HALO_STEP(4) HALO_STEP(2) HALO_STEP(1)
#undef HALO_STEP
#pragma unroll
                for (int b = 0; b < GB; ++b) {
                    const int g = g0 + kWaves * b;
                    if (g < G && lane == 0) {
                        sh.score[g] = p[b];
                        scores[g] = p[b];
                    }
                }
            }
        } else {
            for (int g = wave; g < G; g += kWaves) {
                const float v = dot_order64(h, Bt + (size_t)g * r, r, lane);
                if (lane == 0) {
                    sh.score[g] = v;
                    scores[g] = v;
                }
            }
        }
    } else {
        for (int g = tid; g < G; g += NT) sh.score[g] = scores[g];
    }
    // pad to a multiple of four with NaN: a NaN at an index >= G never ranks before anything
    const int G4 = (G + 3) & ~3;
    if (tid < G4 - G) sh.score[G + tid] = __uint_as_float(0x7fc00000u);
    __syncthreads();

    // rank by counting; thread (g, part) sweeps opponents' float4 pieces q = part, part+P, ...
    const float4 *s4 = reinterpret_cast<const float4 *>(sh.score);
    const int n4 = G4 / 4;
    int P = NT / G;                     // slices per group (>= 1 when G <= NT)
    if (P < 1) P = 1;
    if (P > n4) P = n4;
    for (int base = 0; base < G * P; base += NT) {
        const int idx = base + tid;
        if (idx < G * P) {
            const int g = idx % G, part = idx / G;
            const float sg = sh.score[g];
            int cnt = 0;
            for (int q = part; q < n4; q += P) {
                const float4 v = s4[q];
                cnt += ranks_before(v.x, 4 * q, sg, g) ? 1 : 0;
                cnt += ranks_before(v.y, 4 * q + 1, sg, g) ? 1 : 0;
                cnt += ranks_before(v.z, 4 * q + 2, sg, g) ? 1 : 0;
                cnt += ranks_before(v.w, 4 * q + 3, sg, g) ? 1 : 0;
            }
            if (cnt) atomicAdd(&sh.pos[g], cnt);
        }
    }
    __syncthreads();

    // priority index -> device -> survives?
    for (int g = tid; g < G; g += NT) {
        const int pos = sh.pos[g];
        uint8_t m = 0;
        int dev = -1;
        if (pos < K) {
            dev = sh.prio[pos];
            if (dev >= 0 && dev < n_dev)
                m = sh.drop[dev] ? 0 : 1;
            else
                dev = -1;   // malformed schedule entry: treated as not executed
        }
        if (order) order[pos] = g;
        if (group_dev) group_dev[g] = (int8_t)dev;
        mask[g] = m;
        sh.keep[g] = m;
    }
    __syncthreads();
    // survivors in ascending group order: one ballot word per 64 groups
    for (int g0 = 0; g0 < G; g0 += NT) {          // uniform trip count
        const int g = g0 + tid;
        const unsigned long long b = __ballot(g < G && sh.keep[g]);
        if (lane == 0) sh.bits[(g0 >> 6) + wave] = b;
    }
    __syncthreads();
    const int n_words = (G + 63) >> 6;
    int total = 0;
    for (int j = 0; j < n_words; ++j) total += __popcll(sh.bits[j]);
    if (tid == 0 && n_surv) *n_surv = total;
    if (surv_idx) {
        for (int g = tid; g < G; g += NT) {
            if (!sh.keep[g]) continue;
            const int wd = g >> 6;
            int c = __popcll(sh.bits[wd] & ((1ull << (g & 63)) - 1ull));
            for (int j = 0; j < wd; ++j) c += __popcll(sh.bits[j]);
            surv_idx[c] = g;
        }
        for (int p = total + tid; p < K; p += NT) surv_idx[p] = -1;
    }
}

}  // namespace halo
