// Workgroup-level routine for the Pred step's second half (paper Sec. III-B.2 / III-B.3):
// [optionally the predictor's second layer] -> importance rank -> priority index -> device
// -> surviving set, for ONE token.  Shared by the stand-alone kernels (mask.hip) and by the
// decode kernels that carry the next block's prediction in spare workgroups (ffn_decode.hip).
//
// Ranking by counting: rank(g) = number of groups that come before g under (score
// descending, lower index first on equal scores, NaN after every number).  Every score is
// turned once into a 64-bit key whose unsigned order IS that order (rank_key below), so a
// comparison is one instruction; the G x G comparisons are spread over all threads of the
// workgroup (each thread takes one group and one slice of the opponents; slices are summed
// with LDS atomics).  With float comparisons and the NaN / tie cases decided pair by pair the
// sweep was 650 instructions per wave, a third of the workgroup's whole time.  Survivor
// positions come from wave ballots.
#pragma once
#include "common.hpp"

namespace halo {

// Key of (score s, group g), g < 1024: h comes before g in the ranking exactly when
// rank_key(s_h, h) > rank_key(s_g, g).  High 32 bits: the float's bits made monotonic (sign flipped
// for positives, all bits flipped for negatives), -0 taken as +0 so that the two tie, NaN taken as 0,
// below -inf.  Low 10 bits: 1023 - g, so that among equal scores the lower index is the larger key.
__device__ __forceinline__ unsigned long long rank_key(float s, int g)
{
    uint32_t u = __float_as_uint(s);
    if ((u << 1) == 0u) u = 0u;                                   // -0 -> +0
    uint32_t k = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    if (s != s) k = 0u;                                           // NaN after every number
    return ((unsigned long long)k << 10) | (unsigned)(1023 - g);
}

struct MaskShared {
    __attribute__((aligned(16))) unsigned long long key[1024];
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
    constexpr int GB = 8;                       // slots whose rows a wave fetches before reducing any
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
    // Rows of up to 256 elements occupy half a wave, so a wave takes two at a time: lanes 0..31 row
    // 2s, lanes 32..63 row 2s + 1.  In the fixed order the partial sums of lanes 32..63 are then +0,
    // and the butterfly's first step (distance 32) adds exactly that: here it is `+ 0.0f` in every
    // lane, and the steps at distances 16..1 stay inside a half.  Same bits, half the instructions.
    const bool paired = FUSED && r <= 256;
    const int pl = paired ? (lane & 31) : lane, half = paired ? (lane >> 5) : 0;
    const bool on = pl * 8 < r;
    float hx[8];
    Piece8<WT> w[GB];
    // batch starting at slot s0 of this wave: slot s = s0 + kWaves * b holds row s (or rows 2s, 2s+1)
    auto row_of_slot = [&](int s) { return paired ? 2 * s + half : s; };
    auto load_batch = [&](int s0) {
#pragma unroll
        for (int b = 0; b < GB; ++b) {
            const int g = row_of_slot(s0 + kWaves * b);
            const bool ok = on && g < G;
            w[b].load(Bt + (size_t)(g < G ? g : G - 1) * r + (on ? pl * 8 : 0));
            if (!ok) w[b].zero();
        }
    };
    const int n_slots = paired ? (G + 1) / 2 : G;
    if (fast) {
        // rows first, h last: the lanes outside h are cleared once h has arrived, and a wait for h placed
        // in front of the row requests would make two memory round trips of one
        load_batch(wave < n_slots ? wave : 0);  // a wave beyond the last slot loads (and later discards) batch 0
        load8(h + (on ? pl * 8 : 0), hx);
        if (!on) {
#pragma unroll
            for (int e = 0; e < 8; ++e) hx[e] = 0.0f;
        }
    }
    if (tid < K) sh.prio[tid] = pv;
    for (int p = tid + NT; p < K; p += NT) sh.prio[p] = prio_dev[p];
    if (tid < n_dev) sh.drop[tid] = drop ? dv : 0;
    for (int g = tid; g < 1024; g += NT) sh.pos[g] = 0;
    if (FUSED) {
        if (fast) {
            for (int s0 = wave; s0 < n_slots; s0 += kWaves * GB) {
                if (s0 != wave) load_batch(s0);
                float p[GB];
#pragma unroll
                for (int b = 0; b < GB; ++b) {
                    p[b] = 0.0f;
                    if (s0 + kWaves * b < n_slots) {            // uniform: slots past the end cost nothing
                        float wf[8];
                        w[b].get(wf);
#pragma unroll
                        for (int e = 0; e < 8; ++e) p[b] = __builtin_fmaf(hx[e], wf[e], p[b]);
                    }
                }
                // the butterflies advance together, distance by distance
#define HALO_STEP(OFF)                                           \
    _Pragma("unroll") for (int b = 0; b < GB; ++b) p[b] = xor_add<OFF>(p[b]);
                if (paired) {
#pragma unroll
                    for (int b = 0; b < GB; ++b) p[b] = p[b] + 0.0f;
                } else {
                    HALO_STEP(32)
                }
                HALO_STEP(16) HALO_STEP(8) HALO_STEP(4) HALO_STEP(2) HALO_STEP(1)
#undef HALO_STEP
#pragma unroll
                for (int b = 0; b < GB; ++b) {
                    const int g = row_of_slot(s0 + kWaves * b);
                    if (g < G && pl == 0) {
                        sh.key[g] = rank_key(p[b], g);
                        scores[g] = p[b];
                    }
                }
            }
        } else {
            for (int g = wave; g < G; g += kWaves) {
                const float v = dot_order64(h, Bt + (size_t)g * r, r, lane);
                if (lane == 0) {
                    sh.key[g] = rank_key(v, g);
                    scores[g] = v;
                }
            }
        }
    } else {
        for (int g = tid; g < G; g += NT) sh.key[g] = rank_key(scores[g], g);
    }
    // pad to an even count with key 0, which comes before nothing
    const int G2 = (G + 1) & ~1;
    if (tid < G2 - G) sh.key[G + tid] = 0ull;
    __syncthreads();

    // rank by counting; thread (g, part) sweeps the opponents' keys in pairs q = part, part+P, ...
    const ulonglong2 *k2 = reinterpret_cast<const ulonglong2 *>(sh.key);
    const int n2 = G2 / 2;
    int P = NT / G;                     // slices per group (>= 1 when G <= NT)
    if (P < 1) P = 1;
    if (P > n2) P = n2;
    for (int base = 0; base < G * P; base += NT) {
        const int idx = base + tid;
        if (idx < G * P) {
            const int g = idx % G, part = idx / G;
            const unsigned long long kg = sh.key[g];
            int cnt = 0;
            for (int q = part; q < n2; q += 4 * P) {            // four pairs requested before any is compared
                ulonglong2 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = k2[q + k * P < n2 ? q + k * P : q];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (q + k * P < n2) {
                        cnt += v[k].x > kg ? 1 : 0;
                        cnt += v[k].y > kg ? 1 : 0;
                    }
                }
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
