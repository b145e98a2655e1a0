// Internal launcher interface between the C boundary (halo_api.hip) and the kernels.
#pragma once
#include <hip/hip_ext.h>

#include "common.hpp"

namespace halo {

// predictor.hip
hipError_t launch_predictor(int dtype, const void *x, int T, int d, int r, int G, const void *At,
                            const void *Bt, float *h, float *scores, hipStream_t s);

// mask.hip
hipError_t launch_group_mask(const float *scores, int T, int G, int K, const int8_t *prio_dev,
                             int n_dev, const uint8_t *drop, int32_t *order, int8_t *group_dev,
                             uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s);

hipError_t launch_scores_and_mask(int dtype, const float *h, const void *Bt, int r, float *scores,
                                  int T, int G, int K, const int8_t *prio_dev, int n_dev,
                                  const uint8_t *drop, int32_t *order, int8_t *group_dev,
                                  uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s);

// ffn_decode.hip : float-ALU paths (any T; tuned for one token)
struct DecodeScratch {
    int32_t *ulist;     // [G]   groups surviving for at least one token, ascending
    int32_t *meta;      // meta[0] = number of entries of ulist
    float *act;         // [T][ffn] activations SiLU(gate)*up, compacted by union slot
                        // (the matrix-core paths store bf16 in the same buffer)
    int32_t *tok_list;  // [G][T] prefill: tokens that keep each group, ascending
    int32_t *tok_cnt;   // [G]
    int32_t *slot;      // [T][G] position of the token in its group's list, -1 = not kept
    float *partial;     // [splits][T][d] prefill: the down projection's sums per range of groups
    bf16_t *q4_w = nullptr;   // 4-bit callers with many tokens: room for Wg, Wu [ffn][d] and Wd [G][d][gs] as bf16, or null
};
// The next block's prediction (predictor + mask from x_next), see halo_ffn_forward_ahead.
struct AheadArgs {
    const void *x_next, *At, *Bt;
    int r, K, n_dev;
    const int8_t *prio_dev;
    const uint8_t *drop;
    float *h, *scores;
    int32_t *order;
    int8_t *group_dev;
    uint8_t *mask;
    int32_t *surv_idx, *n_surv;
};
// Arguments of the prediction for the next block that rides along with this block's kernels.
struct AheadDev {
    const float *h;          // [r] first-layer output, written by the gate/up launch
    const bf16_t *Bt;        // [G][r]
    int r, K, n_dev;
    const int8_t *prio_dev;
    const uint8_t *drop;     // [n_dev] or nullptr
    float *scores;           // [G]
    int32_t *order;
    int8_t *group_dev;
    uint8_t *mask;
    int32_t *surv_idx;
    int32_t *n_surv;
};
// The first predictor layer of the next block for T tokens, riding in the first n_pred workgroups of
// a gate/up launch (four rows of At per workgroup): h[t][j] = ReLU(x_next[t] . At[j]).
struct AheadPredDev {
    const bf16_t *x_next, *At;
    float *h;
    int r, n_pred;       // n_pred == 0: nothing rides along
};
inline AheadPredDev ahead_pred_dev(const AheadArgs *a)
{
    if (!a) return AheadPredDev{nullptr, nullptr, nullptr, 0, 0};
    return AheadPredDev{(const bf16_t *)a->x_next, (const bf16_t *)a->At, a->h, a->r, (a->r + 3) / 4};
}
inline AheadDev ahead_dev(const AheadArgs &a)
{
    return AheadDev{a.h, (const bf16_t *)a.Bt, a.r, a.K, a.n_dev, a.prio_dev, a.drop, a.scores, a.order,
                    a.group_dev, a.mask, a.surv_idx, a.n_surv};
}
// the one-token down projection on its own (also the attention block's output projection)
hipError_t launch_down_t1(const bf16_t *Wd, int d, int G, const uint8_t *mask, const bf16_t *act, bf16_t *y,
                          hipStream_t s, const AheadArgs *ahead = nullptr);
hipError_t launch_down_generic_bf16(const float *act, int act_stride, int d, int gs, const bf16_t *Wd,
                                    const int32_t *ulist, const int32_t *meta, bf16_t *y, hipStream_t s);

hipError_t launch_ffn_decode(int dtype, const void *x, int T, int d, int G, int gs, const void *Wg,
                             const void *Wu, const void *Wd, const uint8_t *mask, void *y,
                             const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead = nullptr,
                             bool *ahead_fused = nullptr);

hipError_t launch_union(const uint8_t *mask, int T, int G, int32_t *ulist, int32_t *meta, hipStream_t s);

// ffn_mfma.hip : bf16 matrix-core path for a few tokens (2 <= T <= 16)
bool mfma_path_supported(int T, int d, int gs);
hipError_t launch_ffn_mfma(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                           const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                           const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead = nullptr,
                           bool *ahead_fused = nullptr);

// ffn_few.hip : gate/up for 2..8 tokens on the float ALUs (rows streamed as in the one-token path)
bool few_path_supported(int T, int d, int G, int gs);
hipError_t launch_gate_up_few(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                              const uint8_t *mask, bf16_t *act, int act_stride, hipStream_t s,
                              const AheadPredDev &ap);

// ffn_prefill.hip : bf16 matrix-core path for many tokens
bool prefill_path_supported(int T, int d, int gs);
int prefill_down_splits(int T, int d, int G);   // ranges of groups in the down projection (0: one pass, no ranges)
hipError_t launch_ffn_prefill(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg,
                              const bf16_t *Wu, const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                              const DecodeScratch &ws, hipStream_t s);

// ffn_q4.hip : 4-bit block-quantised weights (blocks of 128 along the reduction dimension)
struct Q4Weights {
    const uint32_t *gate_codes;   // [ffn][d/8]
    const bf16_t *gate_scales;    // [ffn][d/128]
    const uint32_t *up_codes;
    const bf16_t *up_scales;
    const uint32_t *down_codes;   // [G][d][gs/8]
    const bf16_t *down_scales;    // [G][d]
};
bool q4_shape_supported(int d, int gs);
// many tokens over 4-bit weights can run on the bf16 matrix-core kernels once the weights are expanded
bool q4_expand_supported(int T, int dtype, int d, int G, int gs);
// rank: the predictor's size; the few-token kernel shapes its work around the predictor rows it carries when
// one step is overlapped with the next, and shapes it the same way when it carries none (same bits either way)
hipError_t launch_ffn_q4(int dtype, const void *x, int T, int d, int G, int gs, const Q4Weights &w,
                         const uint8_t *mask, void *y, const DecodeScratch &ws, hipStream_t s, int rank,
                         const AheadArgs *ahead = nullptr, bool *ahead_fused = nullptr);

// ffn_q4_mt.hip : 4-bit weights, 2..16 tokens, matrix cores
bool q4_mfma_path_supported(int T, int d, int G, int gs);
hipError_t launch_ffn_q4_mfma(const bf16_t *x, int T, int d, int G, const Q4Weights &w, const uint8_t *mask,
                              bf16_t *y, const DecodeScratch &ws, hipStream_t s, int rank,
                              const AheadArgs *ahead = nullptr, bool *ahead_fused = nullptr);

// mha_decode.hip : head-sparse attention for one new token (bf16, head dimension 128)
struct MhaScratch {
    float *q;            // [H][128] queries of the surviving heads, compact by slot
    float *part;         // [H][chunks][130] partial softmaxes
    DecodeScratch dec;   // ulist / meta / act as in the FFN
};
constexpr int kMhaChunk = 128;
constexpr int kMhaMaxLen = 131072;   // cache rows: 1024 chunks
bool mha_shape_supported(int d, int head_dim);
hipError_t launch_mha_decode(const void *x, int d, int H, const void *Wq, const void *Wk, const void *Wv,
                             const void *Wo, void *k_cache, void *v_cache, int max_len, int pos,
                             const uint8_t *mask, void *y, const MhaScratch &ws, hipStream_t s,
                             const AheadArgs *ahead = nullptr, bool *ahead_fused = nullptr);

// profile.hip : optional HIP-event bracket around the dominant FFN kernel
bool timer_acquire(hipEvent_t *start, hipEvent_t *stop);   // false: not profiling (or pool used up)
void timer_commit(const char *kernel_name);

// Launch `kernel`; while profiling is active its dispatch carries a start/stop event pair, so
// the elapsed time is that of the kernel itself (no launch gap inside the bracket).
template <typename F, typename... Args>
inline void launch_timed_lds(const char *name, F kernel, dim3 grid, dim3 block, size_t lds_bytes,
                             hipStream_t s, Args... args)
{
    hipEvent_t e0, e1;
    if (timer_acquire(&e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, s, e0, e1, 0, args...);
        timer_commit(name);
    } else {
        kernel<<<grid, block, lds_bytes, s>>>(args...);
    }
}

template <typename F, typename... Args>
inline void launch_timed(const char *name, F kernel, dim3 grid, dim3 block, hipStream_t s, Args... args)
{
    launch_timed_lds(name, kernel, grid, block, 0, s, args...);
}

}  // namespace halo
