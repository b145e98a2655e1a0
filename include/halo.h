/*
 * halo.h -- C boundary of the MI355X (gfx950) implementation of HALO's per-token
 * neuron-group-sparse FFN path:  predictor -> group mask -> group-sparse SwiGLU FFN.
 *
 * Conventions (all entry points unless stated otherwise)
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned,
 *     row-major and dense.  The library never allocates or frees device memory:
 *     scratch comes from the caller's `workspace` (size from halo_workspace_bytes).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     validate their arguments on the host, enqueue kernels on that stream and
 *     return without synchronising; HALO_OK means "enqueued".
 *   - On any error nothing is enqueued and no output is touched.  No C++ exception
 *     crosses this boundary.
 *   - Weight element type is given by halo_shape.dtype: HALO_F32 (float) or
 *     HALO_BF16 (bfloat16: the upper 16 bits of an IEEE float, round-to-nearest-even).
 *     Hidden states x and the output y use the same type.  Scores are always float.
 *   - Limits: d % 8 == 0, rank % 8 == 0, ffn == n_groups * group_size,
 *     1 <= n_groups <= 1024, 1 <= n_dev <= 127, T >= 0 (T == 0 is a no-op).
 *
 * Weight layout (the FFN's weights cut into neuron groups, paper Sec. II-A):
 * neuron group g owns rows [g*group_size, (g+1)*group_size) of
 *   Wg [ffn][d]  gate projection,
 *   Wu [ffn][d]  up projection,
 * and block g of
 *   Wd [n_groups][d][group_size]  down projection, group-blocked:
 *                Wd[g][j][m] = weight from neuron g*group_size+m to output j,
 * so one group is three contiguous blocks of group_size*d elements, and within the down
 * block the neurons of the group are contiguous for every output.  (From the usual
 * [d][ffn] down matrix W: Wd = W.view(d, n_groups, group_size).permute(1, 0, 2).)
 */
#ifndef HALO_H
#define HALO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HALO_OK = 0,
    HALO_ERR_NULL = -1,      /* a required pointer is NULL */
    HALO_ERR_SHAPE = -2,     /* shape fields inconsistent or outside the limits */
    HALO_ERR_DTYPE = -3,     /* unknown dtype */
    HALO_ERR_ARG = -4,       /* scalar argument out of range (k_keep, n_dev, T, alignment) */
    HALO_ERR_WORKSPACE = -5, /* workspace NULL or smaller than halo_workspace_bytes */
    HALO_ERR_HIP = -6        /* a HIP runtime call failed (launch error) */
} halo_status;

typedef enum { HALO_F32 = 0, HALO_BF16 = 1 } halo_dtype;

typedef struct {
    int32_t d;          /* hidden dimension D */
    int32_t ffn;        /* FFN intermediate dimension */
    int32_t group_size; /* neurons per group */
    int32_t n_groups;   /* N_g = ffn / group_size */
    int32_t rank;       /* predictor hidden dimension */
    int32_t dtype;      /* halo_dtype */
} halo_shape;

/* Human-readable name of a status code (static string, never NULL). */
const char *halo_status_string(int status);

/*
 * PLR-aware ratio-guided scheduler (paper Alg. 3 and the worked example of
 * Sec. III-B.4).  HOST pointers, no GPU work.
 *   n_prio   number of priority indices to distribute (0 = most significant);
 *            the path uses n_prio = k_keep, i.e. the kept ranks are distributed.
 *   ratios   [n_dev] workload ratios, non-negative (need not be normalised to
 *            rounding error), or NULL for the homogeneous setting 1/n_dev.
 *   plr      [n_dev] packet-loss rates in [0,1].
 *   prio_dev [n_prio] out: device executing priority index p.  Devices are taken
 *            in ascending PLR (ties: lower device index); device k of that order
 *            receives the contiguous run [b_{k-1}, b_k), b_k = floor(n_prio *
 *            (r_1+..+r_k) + 1/2), the last cut forced to n_prio.
 * Errors: HALO_ERR_NULL, HALO_ERR_ARG (n_prio < 0, n_dev outside 1..127, NaN,
 * negative ratio, PLR outside [0,1]).
 */
int halo_build_schedule(int32_t n_prio, int32_t n_dev, const double *ratios,
                        const double *plr, int8_t *prio_dev);

/*
 * Workload ratios from device memory budgets and computing power: the first step of the
 * paper's load-balancing scheduler, whose output feeds halo_build_schedule.  HOST
 * pointers, no GPU work.  mem[i] >= 0 and comp[i] > 0 are device i's memory budget and
 * computing power, demand > 0 is the model's total memory demand M_t (same unit as mem);
 * ratios[n_dev] (out) is non-negative and sums to 1.
 *   halo_ratios_comp_greedy  paper Alg. 1: devices in descending computing power (ties: lower
 *                            index first) are filled to their budget until the demand is
 *                            covered; the last one used takes only the remainder.
 *   halo_ratios_min_max      paper Alg. 2: bisection, until the interval is no wider than eps
 *                            (the paper uses 1e-3), on the threshold T over [0, max(mem)/min(comp)]
 *                            for the smallest T with sum_i min(mem_i, T*comp_i) >= demand; device i
 *                            gets min(mem_i, T*comp_i), normalised.
 * Errors: HALO_ERR_NULL; HALO_ERR_ARG (n_dev outside 1..127, NaN, negative budget, non-positive
 * computing power / demand / eps, or total budget below the demand -- the algorithms' assertion).
 */
int halo_ratios_comp_greedy(int32_t n_dev, const double *mem, const double *comp, double demand,
                            double *ratios);
int halo_ratios_min_max(int32_t n_dev, const double *mem, const double *comp, double demand, double eps,
                        double *ratios);

/*
 * Upper bound, in bytes, of the scratch any entry point below needs for up to T tokens
 * of this shape with k_keep groups kept per token: the value never falls as T grows, so a
 * workspace sized for the largest call serves the smaller ones.  Returns 0 for invalid
 * arguments.
 */
size_t halo_workspace_bytes(const halo_shape *shape, int32_t T, int32_t k_keep);

/*
 * The same, for callers of the `_q4` entry points further down: for more than 16 tokens (bf16) the bound
 * also holds one block's FFN weights as bf16 (3 * ffn * d * 2 bytes).  With that room the 4-bit weights of
 * a many-token call are expanded once into the workspace and the call runs on the bf16 matrix-core
 * kernels; a `_q4` call given only halo_workspace_bytes works all the same and walks the tokens 16 at a
 * time instead (several times slower).  Never smaller than halo_workspace_bytes; 0 for invalid arguments.
 */
size_t halo_workspace_bytes_q4(const halo_shape *shape, int32_t T, int32_t k_keep);

/*
 * Semantic-aware predictor (paper Sec. III-B.2): one significance value per
 * neuron group from the hidden state, through a two-matrix network
 *     h = ReLU(x A),  scores = h B      (A: d x rank, B: rank x n_groups, no bias).
 *   x      [T][d]          hidden states (dtype)
 *   At     [rank][d]       A transposed (dtype)
 *   Bt     [n_groups][rank] B transposed (dtype)
 *   scores [T][n_groups]   out, float
 * Arithmetic is float32 with a fixed summation order so that rankings are
 * reproducible bit for bit: a dot product of length n keeps 64 partial sums,
 * element i going to partial (i/8) mod 64 by fused multiply-add in increasing i
 * from +0; partials are combined pairwise at distances 32,16,8,4,2,1.
 * Uses workspace for h ([T][rank] float).
 */
int halo_predict_scores(const halo_shape *shape, const void *x, int32_t T, const void *At,
                        const void *Bt, float *scores, void *workspace, size_t ws_bytes,
                        void *stream);

/*
 * Importance rank -> priority index -> device -> surviving set (paper Sec. III-B.3:
 * the Pred step's mapping, and the relaxed merge that skips lost uploads).
 *   scores    [T][G] float
 *   k_keep    groups executed per token (0..G): the k_keep highest-scoring groups.
 *             Ranking: score descending, equal scores by lower group index, NaN last.
 *   prio_dev  [k_keep] int8: device executing the group of rank p (from
 *             halo_build_schedule, copied to the device by the caller).  An entry
 *             outside [0, n_dev) makes its group count as not executed
 *             (group_dev -1, mask 0); nothing is read out of bounds.
 *   drop      [T][n_dev] uint8, non-zero = that device's partial result for that
 *             token is lost; NULL = nothing is lost.
 * Outputs (each may be NULL if not wanted, except mask):
 *   order     [T][G] int32  group index at each rank (rank 0 = most significant)
 *   group_dev [T][G] int8   device of each group, -1 if not executed
 *   mask      [T][G] uint8  1 = executed and not lost (survives), else 0
 *   surv_idx  [T][k_keep] int32 surviving group indices ascending, padded with -1
 *   n_surv    [T] int32     number of surviving groups
 */
int halo_build_group_mask(const float *scores, int32_t T, int32_t G, int32_t k_keep,
                          const int8_t *prio_dev, int32_t n_dev, const uint8_t *drop,
                          int32_t *order, int8_t *group_dev, uint8_t *mask,
                          int32_t *surv_idx, int32_t *n_surv, void *stream);

/*
 * Group-sparse SwiGLU FFN (paper Sec. II-A "Neuron group"; merge = plain sum of the
 * groups' partial results, Sec. III-B.3):
 *     y[t][j] = sum_{g : mask[t][g] != 0}  sum_{m < group_size}
 *                   Wd[g][j][m] * SiLU(Wg[g*group_size+m].x[t]) * (Wu[g*group_size+m].x[t])
 * Only groups that survive for at least one token are read from memory; a group
 * with mask 0 contributes exactly zero to that token; a token with no surviving
 * group gets y[t] = 0.
 *   x [T][d], Wg/Wu [ffn][d], Wd [n_groups][d][group_size], mask [T][n_groups] uint8,
 *   y [T][d] out (dtype).
 * Accumulation is float32; the tuned bf16 paths round the activation SiLU(gate)*up to bf16 before
 * the down projection.
 * Which kernels run (results are the same to the stated tolerance either way; throughput is not):
 *   bf16, group size 128, n_groups <= 256, one token, d = 5120 or a multiple of 1024 in [2048, 8192]:
 *       the streaming one-token kernels;
 *   bf16, group size 128, 2..16 tokens, d a multiple of 128: the few-token kernels (2..4 tokens with
 *       d in {4096, 5120, 8192} and n_groups <= 256 on the float ALUs, otherwise matrix cores);
 *   bf16, group size 128, more than 16 tokens, d a multiple of 128: the many-token matrix-core kernels;
 *   anything else (float32, other group sizes or row lengths): plain wave-per-row kernels, several
 *       times slower per byte.
 */
int halo_group_sparse_ffn(const halo_shape *shape, const void *x, int32_t T, const void *Wg,
                          const void *Wu, const void *Wd, const uint8_t *mask, void *y,
                          void *workspace, size_t ws_bytes, void *stream);

/*
 * One whole pass for an FFN block on one stream, no host synchronisation:
 * halo_predict_scores -> halo_build_group_mask -> halo_group_sparse_ffn
 * (paper Sec. III-A generation phase: Pred, Load, Comp and the merge for one block).
 * x_pred is the hidden state the predictor reads ([T][d]; pass x itself to predict
 * from the block's own input, or the previous layer's input for the paper's
 * one-layer-ahead prediction).  Optional outputs (scores, order, group_dev, mask,
 * surv_idx, n_surv) may each be NULL; they are then kept in the workspace.
 */
int halo_ffn_forward(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                     const void *At, const void *Bt, const void *Wg, const void *Wu,
                     const void *Wd, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                     const uint8_t *drop, void *y, float *scores, int32_t *order,
                     int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                     void *workspace, size_t ws_bytes, void *stream);

/*
 * halo_ffn_forward for callers that cannot allocate device memory or hand over a workspace
 * (code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments, results and errors as halo_ffn_forward, without `workspace` / `ws_bytes`.
 * The scratch is a fixed array of halo_static_scratch_bytes() bytes (8 MiB) inside the
 * library's code object; every GPU that runs the library holds its own copy until the process
 * ends.  The call allocates and frees nothing.
 *   - A call whose halo_workspace_bytes(shape, T, k_keep) exceeds that size returns
 *     HALO_ERR_WORKSPACE and enqueues nothing (bf16, d = 4096, 86 groups: up to 47 tokens;
 *     d = 8192, 224 groups: up to 23).
 *   - The first call made with a given device current looks up that device's copy of the array
 *     (a runtime query, no allocation); make that first call outside stream capture.
 *   - All calls on one GPU share the array, which keeps the previous call's contents; nothing
 *     in it has to be cleared (each kernel writes what it later reads).  Calls that overlap on
 *     one GPU -- different streams, or different host threads -- race on it: serialise them.
 */
size_t halo_static_scratch_bytes(void);
int halo_ffn_forward_static(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                            const void *At, const void *Bt, const void *Wg, const void *Wu,
                            const void *Wd, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                            const uint8_t *drop, void *y, float *scores, int32_t *order,
                            int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                            void *stream);

/*
 * Overlapped form of the whole pass (paper Sec. III-B.3 and its figure of the generation
 * phase with overlapped processes: the Pred process for the next block runs beside the
 * Load/Comp of the current one, one layer ahead).  On `stream`:
 *   - group-sparse FFN of the current block, y = FFN(x; mask_cur), with a mask produced by
 *     an earlier call (this one, halo_ffn_forward or halo_build_group_mask);
 *   - predictor + group mask of the next block from x_pred_next with that block's
 *     predictor weights -> mask_next (and the optional outputs, same meaning as in
 *     halo_build_group_mask; NULL = not produced).
 * For one token (bf16, group size 128, n_groups <= 256, d = 5120 or a multiple of 1024 from 2048 to
 * 8192) and for 2..16 tokens (bf16, d a multiple of 128, group size 128, n_groups <= 256) the
 * prediction occupies spare
 * workgroups of the FFN's own two launches (first predictor layer beside gate/up, second
 * layer + ranking + mask beside the down projection), so it costs no launch and little or no
 * time on the critical path; for other shapes it is enqueued after the FFN.  Results are
 * identical to the separate calls either way.  x_pred_next may be x (predicting from this
 * block's input, as the paper does) but must not be y; mask_next must not alias mask_cur.
 */
int halo_ffn_forward_ahead(const halo_shape *shape, const void *x, int32_t T, const void *Wg,
                           const void *Wu, const void *Wd, const uint8_t *mask_cur, void *y,
                           const void *x_pred_next, const void *At_next, const void *Bt_next,
                           int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                           const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                           int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                           int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream);

/*
 * The FFN over 4-bit block-quantised weights (paper Sec. V-A: the evaluated models are
 * quantised to 4-bit integers; the paper fixes no storage format, this one is the library's).
 *
 * Format: blocks of 128 consecutive elements along the reduction dimension share one bf16
 * scale s; an element is s * (c - 8) with a 4-bit code c in 0..15.  Codes are packed eight per
 * 32-bit little-endian word: of the word's eight consecutive elements, element 2i sits in
 * bits [4i, 4i+3] and element 2i+1 in bits [16+4i, 16+4i+3] (i = 0..3).
 *   Wg_codes, Wu_codes : [ffn][d/8] words       Wg_scales, Wu_scales : [ffn][d/128] bf16
 *                        (row m = neuron m, blocks along d)
 *   Wd_codes           : [n_groups][d][16] words Wd_scales           : [n_groups][d] bf16
 *                        (group-blocked like Wd above: the block of output j in group g is
 *                         the group's 128 neurons)
 * Needs group_size == 128 and d % 128 == 0 (HALO_ERR_SHAPE otherwise); shape->dtype is the type
 * of x, y and the predictor weights.  All pointers are device pointers, 16-byte aligned.
 * Everything else -- mask semantics, workspace, stream, errors -- is as in
 * halo_group_sparse_ffn / halo_ffn_forward.  Tuned paths (bf16 activations, n_groups <= 256): one
 * token with d in {4096, 8192} (every surviving code byte streamed once, float ALUs), and 2..16
 * tokens with d a multiple of 1024 up to 8192 (matrix cores, codes expanded in registers); other
 * shapes and float32 activations take a plain path that dequantises element by element.  More than
 * 16 tokens (same shapes): with a workspace of halo_workspace_bytes_q4 the weights are expanded to bf16
 * (each value s * (c - 8) rounded to bf16, to nearest even) and the bf16 kernels of
 * halo_group_sparse_ffn run on them; with less, the 2..16-token kernels walk the tokens 16 at a time.
 */
int halo_group_sparse_ffn_q4(const halo_shape *shape, const void *x, int32_t T, const void *Wg_codes,
                             const void *Wg_scales, const void *Wu_codes, const void *Wu_scales,
                             const void *Wd_codes, const void *Wd_scales, const uint8_t *mask, void *y,
                             void *workspace, size_t ws_bytes, void *stream);

int halo_ffn_forward_q4(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                        const void *At, const void *Bt, const void *Wg_codes, const void *Wg_scales,
                        const void *Wu_codes, const void *Wu_scales, const void *Wd_codes,
                        const void *Wd_scales, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                        const uint8_t *drop, void *y, float *scores, int32_t *order, int8_t *group_dev,
                        uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, void *workspace, size_t ws_bytes,
                        void *stream);

/* halo_ffn_forward_ahead over 4-bit weights: same contract, same weight arguments as
 * halo_group_sparse_ffn_q4.  The prediction rides in spare workgroups on the tuned paths named
 * there; otherwise it is enqueued after the FFN. */
int halo_ffn_forward_ahead_q4(const halo_shape *shape, const void *x, int32_t T, const void *Wg_codes,
                              const void *Wg_scales, const void *Wu_codes, const void *Wu_scales,
                              const void *Wd_codes, const void *Wd_scales, const uint8_t *mask_cur, void *y,
                              const void *x_pred_next, const void *At_next, const void *Bt_next,
                              int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                              const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                              int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                              int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream);

/*
 * The attention block as neuron groups (paper Sec. II-A: a head together with its slice of the
 * output projection forms one group; the block output is the sum of the groups' partial
 * results).  One new token of one sequence (decode) at position pos, 0-based:
 *   every head h    : k_h = Wk_h x, v_h = Wv_h x are written to row pos of the caches -- every
 *                     device keeps the full KV cache (Sec. III-B.3), so keys and values exist
 *                     for every head whether or not its output takes part in the merge;
 *   surviving heads : q_h = Wq_h x,  p = softmax(q_h K_h^T / sqrt(head_dim)) over rows 0..pos,
 *                     o_h = p V_h,  y = sum over surviving h of Wo_h o_h.
 * Plain scaled dot-product attention: no positional rotation, no biases (the paper discusses
 * neither).  Only surviving heads' query rows, cache rows and output-projection blocks are read.
 *
 * halo_mha_shape: d, n_heads (<= 256), head_dim (must be 128), rank of the head predictor,
 * dtype (HALO_BF16 only).  Layouts (device pointers, 16-byte aligned, dense):
 *   x [d], y [d];  Wq, Wk, Wv [n_heads*head_dim][d] (rows of head h contiguous);
 *   Wo head-blocked [n_heads][d][head_dim] (the layout of Wd with heads as groups);
 *   k_cache, v_cache [n_heads][max_len][head_dim], rows 0..pos-1 valid on entry, row pos written;
 *   mask [n_heads] as produced by halo_build_group_mask with G = n_heads.
 * halo_mha_forward runs predictor -> mask -> attention on one stream; the predictor is the same
 * two-matrix network with one output per head (At [rank][d], Bt [n_heads][rank]) and the optional
 * outputs have the meaning they have in halo_ffn_forward.
 * halo_mha_forward_ahead is the overlapped form (same contract as halo_ffn_forward_ahead):
 * attention of the current block with mask_cur, and beside it predictor + head mask of the next
 * block from x_pred_next; for d in {4096, 5120, 8192} the prediction rides in spare workgroups of
 * the q/k/v launch and of the output-projection launch, otherwise it is enqueued afterwards.
 * Errors: as halo_group_sparse_ffn, plus HALO_ERR_ARG for pos outside [0, max_len) or
 * max_len > 131072.
 */
typedef struct {
    int32_t d, n_heads, head_dim, rank;
    int32_t dtype;
} halo_mha_shape;

size_t halo_mha_workspace_bytes(const halo_mha_shape *shape, int32_t max_len);

int halo_head_sparse_mha(const halo_mha_shape *shape, const void *x, const void *Wq, const void *Wk,
                         const void *Wv, const void *Wo, void *k_cache, void *v_cache, int32_t max_len,
                         int32_t pos, const uint8_t *mask, void *y, void *workspace, size_t ws_bytes,
                         void *stream);

int halo_mha_forward(const halo_mha_shape *shape, const void *x, const void *x_pred, const void *At,
                     const void *Bt, const void *Wq, const void *Wk, const void *Wv, const void *Wo,
                     void *k_cache, void *v_cache, int32_t max_len, int32_t pos, int32_t k_keep,
                     const int8_t *prio_dev, int32_t n_dev, const uint8_t *drop, void *y, float *scores,
                     int32_t *order, int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                     void *workspace, size_t ws_bytes, void *stream);

int halo_mha_forward_ahead(const halo_mha_shape *shape, const void *x, const void *Wq, const void *Wk,
                           const void *Wv, const void *Wo, void *k_cache, void *v_cache, int32_t max_len,
                           int32_t pos, const uint8_t *mask_cur, void *y, const void *x_pred_next,
                           const void *At_next, const void *Bt_next, int32_t k_keep, const int8_t *prio_dev,
                           int32_t n_dev, const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                           int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                           int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream);

/*
 * Benchmark aid (not part of the paper's method).  Between halo_profile_begin and
 * halo_profile_end every call of halo_group_sparse_ffn / halo_ffn_forward brackets the
 * FFN's dominant kernel -- the gate/up projection, which streams two thirds of the
 * surviving groups' weight bytes -- with a pair of HIP events on the launch stream.
 * halo_profile_end waits for the recorded events and returns the summed elapsed time
 * (milliseconds), the number of launches timed, and the kernel's name (HOST pointers;
 * each may be NULL).  One launch in `every` is timed (an event-carrying launch costs the
 * host several times a plain one, so timing every launch can leave the GPU waiting for the
 * host and change what is measured), at most max_launches in total.  Do not use while a
 * stream is being captured into a graph.  Errors: HALO_ERR_ARG (bad count or stride, begin
 * while active, end while inactive), HALO_ERR_HIP.
 */
int halo_profile_begin(int32_t max_launches, int32_t every);
int halo_profile_end(double *total_ms, int64_t *launches, char *kernel_name, int32_t name_cap);

/*
 * Harness aid (not part of the paper's method): the glue between the blocks of an FFN-only stack,
 * one launch per layer:  h[t] += y[t] (skipped if y is NULL);  x[t] = h[t] / sqrt(mean(h[t]^2) + eps).
 *   h [T][d] float (in/out, the residual stream), y [T][d] (dtype) or NULL, x [T][d] (dtype) out.
 * d must be a multiple of 4, at most 8192; rows 16-byte aligned.
 * Errors: HALO_ERR_NULL, HALO_ERR_DTYPE, HALO_ERR_ARG (T < 0, d outside those limits, eps < 0), HALO_ERR_HIP.
 */
int halo_stack_residual_norm(float *h, const void *y, void *x, int32_t T, int32_t d, int32_t dtype,
                             float eps, void *stream);

/*
 * Benchmark aids (not part of the paper's method): what this GPU itself sustains for the two
 * resources the path is priced against.  Both enqueue their kernels on `stream`, time them with a
 * HIP event pair and WAIT for the result; results go to HOST pointers (each may be NULL).
 *   halo_peak_read_stream  reads `launches` windows of window_bytes (rounded down to whole 16 KiB
 *       runs) from the device buffer buf, one kernel launch per window, consecutive launches on
 *       consecutive windows of the buffer (wrapping round), with the access pattern of the
 *       one-token gate/up kernel.  gbps = bytes read / elapsed time, launch gaps included, so a
 *       window of a kernel's own size gives what a launch of that size can reach, and a large
 *       window the ceiling of the stream itself.  buf is only read; sink is 4 bytes of device
 *       memory that are practically never written.
 *   halo_peak_mfma_bf16    `launches` launches of a kernel that issues iters * 16 bf16 16x16x32
 *       matrix instructions per wave (eight waves on every compute unit) on non-zero operands;
 *       tflops = multiply-adds * 2 / elapsed time.  sink: 256 bytes of device memory.
 * Errors: HALO_ERR_NULL, HALO_ERR_ARG (misaligned buf, window larger than the buffer or smaller
 * than 16 KiB, counts out of range), HALO_ERR_HIP.
 */
int halo_peak_read_stream(const void *buf, size_t buf_bytes, size_t window_bytes, int32_t launches,
                          void *sink, void *stream, double *gbps, double *us_per_launch);
int halo_peak_mfma_bf16(int32_t iters, int32_t launches, void *sink, void *stream, double *tflops);

#ifdef __cplusplus
}
#endif
#endif /* HALO_H */
