// C boundary of the library: argument validation, workspace carving, kernel enqueue.
// See include/halo.h for the contract of every entry point.
#include "../../include/halo.h"

#include <cmath>
#include <mutex>

#include "kernels.hpp"

// Scratch of halo_ffn_forward_static: one array per GPU the library's code object is loaded on,
// held until the process ends.  The name is only a host-side handle: host code never passes it to
// a kernel, it asks the runtime for the array's device address once per device (scratch_of).
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace halo;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

int check_shape(const halo_shape *s)
{
    if (!s) return HALO_ERR_NULL;
    if (s->dtype != HALO_F32 && s->dtype != HALO_BF16) return HALO_ERR_DTYPE;
    if (s->d < 8 || s->d % 8 || s->rank < 8 || s->rank % 8) return HALO_ERR_SHAPE;
    if (s->group_size < 1 || s->n_groups < 1 || s->n_groups > 1024) return HALO_ERR_SHAPE;
    if ((long long)s->n_groups * s->group_size != (long long)s->ffn) return HALO_ERR_SHAPE;
    return HALO_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Carves the caller's workspace.  The same routine sizes it (base == nullptr).
struct Workspace {
    float *h = nullptr;
    float *scores = nullptr;
    int32_t *order = nullptr;
    int8_t *group_dev = nullptr;
    uint8_t *mask = nullptr;
    int32_t *surv_idx = nullptr;
    int32_t *n_surv = nullptr;
    DecodeScratch dec{};
    size_t bytes = 0;

    // q4_room: also room for one block's weights as bf16 (the 4-bit entry points with many tokens)
    Workspace(const halo_shape &s, int T, int K, void *base, bool q4_room = false)
    {
        char *p = static_cast<char *>(base);
        size_t off = 0;
        auto take = [&](size_t n) -> char * {
            char *r = p ? p + off : nullptr;
            off += align_up(n ? n : 1);
            return r;
        };
        const size_t t = (size_t)(T > 0 ? T : 1), G = (size_t)s.n_groups;
        h = reinterpret_cast<float *>(take(t * s.rank * sizeof(float)));
        scores = reinterpret_cast<float *>(take(t * G * sizeof(float)));
        order = reinterpret_cast<int32_t *>(take(t * G * sizeof(int32_t)));
        group_dev = reinterpret_cast<int8_t *>(take(t * G));
        mask = reinterpret_cast<uint8_t *>(take(t * G));
        surv_idx = reinterpret_cast<int32_t *>(take(t * (size_t)(K > 0 ? K : 1) * sizeof(int32_t)));
        n_surv = reinterpret_cast<int32_t *>(take(t * sizeof(int32_t)));
        dec.ulist = reinterpret_cast<int32_t *>(take(G * sizeof(int32_t)));
        dec.meta = reinterpret_cast<int32_t *>(take(256 * sizeof(int32_t)));
        dec.act = reinterpret_cast<float *>(take(t * (size_t)s.ffn * sizeof(float)));
        dec.tok_list = reinterpret_cast<int32_t *>(take(G * t * sizeof(int32_t)));
        dec.tok_cnt = reinterpret_cast<int32_t *>(take(G * sizeof(int32_t)));
        dec.slot = reinterpret_cast<int32_t *>(take(G * t * sizeof(int32_t)));
        // partial sums of the prefill down projection: the number of ranges falls as T grows, so the
        // size is taken as the largest need of any token count up to T (a workspace sized for T then
        // also serves every smaller call); the need is largest at the upper end of a token tile
        size_t partial_elems = 0;
        if (s.dtype == HALO_BF16) {
            for (int t1 = 256; t1 - 256 < T; t1 += 256) {
                const int tt = t1 < T ? t1 : T;
                if (!prefill_path_supported(tt, s.d, s.group_size) || mfma_path_supported(tt, s.d, s.group_size))
                    continue;
                const int splits = prefill_down_splits(tt, s.d, s.n_groups);
                const size_t need = splits > 1 ? (size_t)splits * tt * s.d : 0;
                partial_elems = need > partial_elems ? need : partial_elems;
            }
        }
        dec.partial = reinterpret_cast<float *>(take(partial_elems * sizeof(float)));
        // appended last: the layout in front of it is the same with and without
        if (q4_room && q4_expand_supported(T, s.dtype, s.d, s.n_groups, s.group_size))
            dec.q4_w = reinterpret_cast<bf16_t *>(take((size_t)3 * s.ffn * s.d * sizeof(bf16_t)));
        bytes = off;
    }
};

int check_mha_shape(const halo_mha_shape *s)
{
    if (!s) return HALO_ERR_NULL;
    if (s->dtype != HALO_BF16) return HALO_ERR_DTYPE;
    if (s->d < 8 || s->d % 8 || s->rank < 8 || s->rank % 8) return HALO_ERR_SHAPE;
    if (s->n_heads < 1 || s->n_heads > 256 || !mha_shape_supported(s->d, s->head_dim)) return HALO_ERR_SHAPE;
    return HALO_OK;
}

// The attention block's workspace: the FFN's carving with heads as groups, plus queries and
// partial softmaxes.
struct MhaWorkspace {
    halo_shape as_ffn{};
    Workspace base;
    MhaScratch mha{};
    size_t bytes = 0;

    static halo_shape ffn_view(const halo_mha_shape &s)
    {
        halo_shape f{};
        f.d = s.d;
        f.ffn = s.n_heads * s.head_dim;
        f.group_size = s.head_dim;
        f.n_groups = s.n_heads;
        f.rank = s.rank;
        f.dtype = (halo_dtype)s.dtype;
        return f;
    }

    MhaWorkspace(const halo_mha_shape &s, int max_len, void *p)
        : as_ffn(ffn_view(s)), base(as_ffn, 1, s.n_heads, p)
    {
        size_t off = base.bytes;
        char *b = static_cast<char *>(p);
        auto take = [&](size_t n) -> char * {
            char *r = b ? b + off : nullptr;
            off += align_up(n);
            return r;
        };
        const size_t chunks = (size_t)(max_len + kMhaChunk - 1) / kMhaChunk;
        mha.q = reinterpret_cast<float *>(take((size_t)s.n_heads * s.head_dim * sizeof(float)));
        mha.part = reinterpret_cast<float *>(take((size_t)s.n_heads * chunks * (s.head_dim + 2) * sizeof(float)));
        mha.dec = base.dec;
        bytes = off;
    }
};

// Device address of `scratch` on the current device (each GPU has its own copy at its own
// address), resolved on the first call made with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

int scratch_of(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HALO_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HALO_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return HALO_OK;
}

}  // namespace

extern "C" {

const char *halo_status_string(int status)
{
    switch (status) {
    case HALO_OK: return "ok";
    case HALO_ERR_NULL: return "required pointer is NULL";
    case HALO_ERR_SHAPE: return "inconsistent or unsupported shape";
    case HALO_ERR_DTYPE: return "unknown dtype";
    case HALO_ERR_ARG: return "argument out of range";
    case HALO_ERR_WORKSPACE: return "workspace missing or too small";
    case HALO_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int halo_build_schedule(int32_t n_prio, int32_t n_dev, const double *ratios, const double *plr,
                        int8_t *prio_dev)
{
    if (!plr || (n_prio > 0 && !prio_dev)) return HALO_ERR_NULL;
    if (n_prio < 0 || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    for (int i = 0; i < n_dev; ++i) {
        if (std::isnan(plr[i]) || plr[i] < 0.0 || plr[i] > 1.0) return HALO_ERR_ARG;
        if (ratios && (std::isnan(ratios[i]) || ratios[i] < 0.0)) return HALO_ERR_ARG;
    }
    // devices in ascending PLR, ties by index: the position of device i is the number
    // of devices that precede it in that order
    int sorted[127];
    for (int i = 0; i < n_dev; ++i) {
        int pos = 0;
        for (int j = 0; j < n_dev; ++j)
            if (plr[j] < plr[i] || (plr[j] == plr[i] && j < i)) ++pos;
        sorted[pos] = i;
    }
    long long begin = 0;
    double cumulative = 0.0;
    for (int k = 0; k < n_dev; ++k) {
        long long end;
        if (k + 1 == n_dev) {
            end = n_prio;
        } else if (!ratios) {
            end = (2LL * n_prio * (k + 1) + n_dev) / (2LL * n_dev);
        } else {
            cumulative += ratios[sorted[k]];
            volatile double scaled = (double)n_prio * cumulative;   // keep multiply and add unfused
            end = (long long)std::floor(scaled + 0.5);
        }
        if (end > n_prio) end = n_prio;
        if (end < begin) end = begin;
        for (long long p = begin; p < end; ++p) prio_dev[p] = (int8_t)sorted[k];
        begin = end;
    }
    return HALO_OK;
}

int halo_ratios_comp_greedy(int32_t n_dev, const double *mem, const double *comp, double demand,
                            double *ratios)
{
    if (!mem || !comp || !ratios) return HALO_ERR_NULL;
    if (n_dev < 1 || n_dev > 127 || !(demand > 0.0)) return HALO_ERR_ARG;
    double budget = 0.0;
    for (int i = 0; i < n_dev; ++i) {
        if (std::isnan(mem[i]) || mem[i] < 0.0 || std::isnan(comp[i]) || comp[i] <= 0.0) return HALO_ERR_ARG;
        budget += mem[i];
    }
    if (budget < demand) return HALO_ERR_ARG;
    // fastest first; equal computing power keeps the lower device index first
    int by_speed[127];
    for (int i = 0; i < n_dev; ++i) {
        int pos = 0;
        for (int j = 0; j < n_dev; ++j)
            if (comp[j] > comp[i] || (comp[j] == comp[i] && j < i)) ++pos;
        by_speed[pos] = i;
    }
    for (int i = 0; i < n_dev; ++i) ratios[i] = 0.0;
    double placed = 0.0;
    for (int k = 0; k < n_dev; ++k) {
        const int dev = by_speed[k];
        if (placed + mem[dev] >= demand) {      // this device completes the demand: it takes the rest
            ratios[dev] = demand - placed;
            break;
        }
        ratios[dev] = mem[dev];
        placed += mem[dev];
    }
    double sum = 0.0;
    for (int i = 0; i < n_dev; ++i) sum += ratios[i];
    for (int i = 0; i < n_dev; ++i) ratios[i] /= sum;
    return HALO_OK;
}

int halo_ratios_min_max(int32_t n_dev, const double *mem, const double *comp, double demand, double eps,
                        double *ratios)
{
    if (!mem || !comp || !ratios) return HALO_ERR_NULL;
    if (n_dev < 1 || n_dev > 127 || !(demand > 0.0) || !(eps > 0.0)) return HALO_ERR_ARG;
    double budget = 0.0, mem_max = 0.0, comp_min = 0.0;
    for (int i = 0; i < n_dev; ++i) {
        if (std::isnan(mem[i]) || mem[i] < 0.0 || std::isnan(comp[i]) || comp[i] <= 0.0) return HALO_ERR_ARG;
        budget += mem[i];
        mem_max = i == 0 ? mem[i] : std::fmax(mem_max, mem[i]);
        comp_min = i == 0 ? comp[i] : std::fmin(comp_min, comp[i]);
    }
    if (budget < demand) return HALO_ERR_ARG;
    // Device i can take min(mem_i, T comp_i) when every device may work for time T; that sum grows
    // with T, and the wanted T is the smallest one at which it reaches the demand.  `hi` always meets
    // the demand (at mem_max / comp_min every device is at its budget), `lo` never does (or is 0);
    // the bracket is halved until it is no wider than eps and its upper end is the answer.
    auto short_of_demand = [&](double t) {
        double taken = 0.0;
        for (int i = 0; i < n_dev; ++i) taken += std::fmin(mem[i], t * comp[i]);
        return taken < demand;
    };
    double lo = 0.0, hi = mem_max / comp_min;
    while (hi - lo > eps) {
        const double mid = (lo + hi) / 2.0;
        (short_of_demand(mid) ? lo : hi) = mid;
    }
    double sum = 0.0;
    for (int i = 0; i < n_dev; ++i) {
        ratios[i] = std::fmin(mem[i], hi * comp[i]);
        sum += ratios[i];
    }
    for (int i = 0; i < n_dev; ++i) ratios[i] /= sum;
    return HALO_OK;
}

size_t halo_workspace_bytes(const halo_shape *shape, int32_t T, int32_t k_keep)
{
    if (check_shape(shape) != HALO_OK || T < 0 || k_keep < 0 || k_keep > shape->n_groups) return 0;
    return Workspace(*shape, T, k_keep, nullptr).bytes;
}

size_t halo_workspace_bytes_q4(const halo_shape *shape, int32_t T, int32_t k_keep)
{
    if (check_shape(shape) != HALO_OK || T < 0 || k_keep < 0 || k_keep > shape->n_groups) return 0;
    return Workspace(*shape, T, k_keep, nullptr, true).bytes;
}

// the workspace of a 4-bit call: with the room for expanded weights when the caller gave that much
static Workspace q4_workspace(const halo_shape &s, int T, int K, void *base, size_t ws_bytes)
{
    Workspace big(s, T, K, base, true);
    return ws_bytes >= big.bytes ? big : Workspace(s, T, K, base);
}

int halo_predict_scores(const halo_shape *shape, const void *x, int32_t T, const void *At,
                        const void *Bt, float *scores, void *workspace, size_t ws_bytes,
                        void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !At || !Bt || !scores) return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(At) || misaligned(Bt) || misaligned(scores)) return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws(*shape, T, 0, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipError_t e = launch_predictor(shape->dtype, x, T, shape->d, shape->rank, shape->n_groups, At, Bt,
                                    ws.h, scores, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_build_group_mask(const float *scores, int32_t T, int32_t G, int32_t k_keep,
                          const int8_t *prio_dev, int32_t n_dev, const uint8_t *drop,
                          int32_t *order, int8_t *group_dev, uint8_t *mask, int32_t *surv_idx,
                          int32_t *n_surv, void *stream)
{
    if (G < 1 || G > 1024) return HALO_ERR_SHAPE;
    if (T < 0 || k_keep < 0 || k_keep > G || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!scores || !mask || (k_keep > 0 && !prio_dev)) return HALO_ERR_NULL;
    hipError_t e = launch_group_mask(scores, T, G, k_keep, prio_dev, n_dev, drop, order, group_dev,
                                     mask, surv_idx, n_surv, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_group_sparse_ffn(const halo_shape *shape, const void *x, int32_t T, const void *Wg,
                          const void *Wu, const void *Wd, const uint8_t *mask, void *y,
                          void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !Wg || !Wu || !Wd || !mask || !y) return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(Wg) || misaligned(Wu) || misaligned(Wd) || misaligned(y))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws(*shape, T, 0, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipError_t e = launch_ffn_decode(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size,
                                     Wg, Wu, Wd, mask, y, ws.dec, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_ffn_forward(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                     const void *At, const void *Bt, const void *Wg, const void *Wu,
                     const void *Wd, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                     const uint8_t *drop, void *y, float *scores, int32_t *order,
                     int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                     void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0 || k_keep < 0 || k_keep > shape->n_groups || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !x_pred || !At || !Bt || !Wg || !Wu || !Wd || !y || (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(x_pred) || misaligned(At) || misaligned(Bt) || misaligned(Wg) ||
        misaligned(Wu) || misaligned(Wd) || misaligned(y) || (scores && misaligned(scores)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws(*shape, T, k_keep, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores ? scores : ws.scores;
    uint8_t *mk = mask ? mask : ws.mask;
    // first predictor layer, then the second layer fused with the ranking / mask kernel
    hipError_t e = launch_predictor(shape->dtype, x_pred, T, shape->d, shape->rank, shape->n_groups,
                                    At, Bt, ws.h, nullptr, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    e = launch_scores_and_mask(shape->dtype, ws.h, Bt, shape->rank, sc, T, shape->n_groups, k_keep,
                               prio_dev, n_dev, drop, order, group_dev, mk, surv_idx, n_surv, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    e = launch_ffn_decode(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size, Wg, Wu,
                          Wd, mk, y, ws.dec, s);
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

size_t halo_static_scratch_bytes(void) { return kStaticScratchBytes; }

int halo_ffn_forward_static(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                            const void *At, const void *Bt, const void *Wg, const void *Wu,
                            const void *Wd, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                            const uint8_t *drop, void *y, float *scores, int32_t *order,
                            int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                            void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0 || k_keep < 0 || k_keep > shape->n_groups || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    // the need is known from the arguments alone: a call that does not fit is refused before anything runs
    if (Workspace(*shape, T, k_keep, nullptr).bytes > kStaticScratchBytes) return HALO_ERR_WORKSPACE;
    if (T == 0) return HALO_OK;
    void *ws = nullptr;
    rc = scratch_of(&ws);
    if (rc) return rc;
    // every kernel of the pass writes the part of the scratch it later reads, so nothing has to be
    // cleared between calls; the kernels take the address like any caller's workspace
    return halo_ffn_forward(shape, x, x_pred, T, At, Bt, Wg, Wu, Wd, k_keep, prio_dev, n_dev, drop, y, scores,
                            order, group_dev, mask, surv_idx, n_surv, ws, kStaticScratchBytes, stream);
}

int halo_group_sparse_ffn_q4(const halo_shape *shape, const void *x, int32_t T, const void *Wg_codes,
                             const void *Wg_scales, const void *Wu_codes, const void *Wu_scales,
                             const void *Wd_codes, const void *Wd_scales, const uint8_t *mask, void *y,
                             void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!q4_shape_supported(shape->d, shape->group_size)) return HALO_ERR_SHAPE;
    if (T < 0) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !Wg_codes || !Wg_scales || !Wu_codes || !Wu_scales || !Wd_codes || !Wd_scales || !mask || !y)
        return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(Wg_codes) || misaligned(Wg_scales) || misaligned(Wu_codes) ||
        misaligned(Wu_scales) || misaligned(Wd_codes) || misaligned(Wd_scales) || misaligned(y))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws = q4_workspace(*shape, T, 0, workspace, ws_bytes);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    const Q4Weights w{(const uint32_t *)Wg_codes, (const bf16_t *)Wg_scales, (const uint32_t *)Wu_codes,
                      (const bf16_t *)Wu_scales, (const uint32_t *)Wd_codes, (const bf16_t *)Wd_scales};
    hipError_t e = launch_ffn_q4(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size, w, mask, y,
                                 ws.dec, static_cast<hipStream_t>(stream), shape->rank);
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_ffn_forward_q4(const halo_shape *shape, const void *x, const void *x_pred, int32_t T,
                        const void *At, const void *Bt, const void *Wg_codes, const void *Wg_scales,
                        const void *Wu_codes, const void *Wu_scales, const void *Wd_codes,
                        const void *Wd_scales, int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                        const uint8_t *drop, void *y, float *scores, int32_t *order, int8_t *group_dev,
                        uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, void *workspace, size_t ws_bytes,
                        void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!q4_shape_supported(shape->d, shape->group_size)) return HALO_ERR_SHAPE;
    if (T < 0 || k_keep < 0 || k_keep > shape->n_groups || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !x_pred || !At || !Bt || !Wg_codes || !Wg_scales || !Wu_codes || !Wu_scales || !Wd_codes ||
        !Wd_scales || !y || (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(x_pred) || misaligned(At) || misaligned(Bt) || misaligned(Wg_codes) ||
        misaligned(Wg_scales) || misaligned(Wu_codes) || misaligned(Wu_scales) || misaligned(Wd_codes) ||
        misaligned(Wd_scales) || misaligned(y) || (scores && misaligned(scores)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws = q4_workspace(*shape, T, k_keep, workspace, ws_bytes);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores ? scores : ws.scores;
    uint8_t *mk = mask ? mask : ws.mask;
    hipError_t e = launch_predictor(shape->dtype, x_pred, T, shape->d, shape->rank, shape->n_groups, At, Bt,
                                    ws.h, nullptr, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    e = launch_scores_and_mask(shape->dtype, ws.h, Bt, shape->rank, sc, T, shape->n_groups, k_keep, prio_dev,
                               n_dev, drop, order, group_dev, mk, surv_idx, n_surv, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    const Q4Weights w{(const uint32_t *)Wg_codes, (const bf16_t *)Wg_scales, (const uint32_t *)Wu_codes,
                      (const bf16_t *)Wu_scales, (const uint32_t *)Wd_codes, (const bf16_t *)Wd_scales};
    e = launch_ffn_q4(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size, w, mk, y, ws.dec, s,
                      shape->rank);
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

size_t halo_mha_workspace_bytes(const halo_mha_shape *shape, int32_t max_len)
{
    if (check_mha_shape(shape) != HALO_OK || max_len < 1 || max_len > kMhaMaxLen) return 0;
    return MhaWorkspace(*shape, max_len, nullptr).bytes;
}

int halo_head_sparse_mha(const halo_mha_shape *shape, const void *x, const void *Wq, const void *Wk,
                         const void *Wv, const void *Wo, void *k_cache, void *v_cache, int32_t max_len,
                         int32_t pos, const uint8_t *mask, void *y, void *workspace, size_t ws_bytes,
                         void *stream)
{
    int rc = check_mha_shape(shape);
    if (rc) return rc;
    if (max_len < 1 || max_len > kMhaMaxLen || pos < 0 || pos >= max_len) return HALO_ERR_ARG;
    if (!x || !Wq || !Wk || !Wv || !Wo || !k_cache || !v_cache || !mask || !y) return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(Wq) || misaligned(Wk) || misaligned(Wv) || misaligned(Wo) ||
        misaligned(k_cache) || misaligned(v_cache) || misaligned(y))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    MhaWorkspace ws(*shape, max_len, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipError_t e = launch_mha_decode(x, shape->d, shape->n_heads, Wq, Wk, Wv, Wo, k_cache, v_cache, max_len, pos,
                                     mask, y, ws.mha, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_mha_forward(const halo_mha_shape *shape, const void *x, const void *x_pred, const void *At,
                     const void *Bt, const void *Wq, const void *Wk, const void *Wv, const void *Wo,
                     void *k_cache, void *v_cache, int32_t max_len, int32_t pos, int32_t k_keep,
                     const int8_t *prio_dev, int32_t n_dev, const uint8_t *drop, void *y, float *scores,
                     int32_t *order, int8_t *group_dev, uint8_t *mask, int32_t *surv_idx, int32_t *n_surv,
                     void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_mha_shape(shape);
    if (rc) return rc;
    if (max_len < 1 || max_len > kMhaMaxLen || pos < 0 || pos >= max_len || k_keep < 0 ||
        k_keep > shape->n_heads || n_dev < 1 || n_dev > 127)
        return HALO_ERR_ARG;
    if (!x || !x_pred || !At || !Bt || !Wq || !Wk || !Wv || !Wo || !k_cache || !v_cache || !y ||
        (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (misaligned(x) || misaligned(x_pred) || misaligned(At) || misaligned(Bt) || misaligned(Wq) ||
        misaligned(Wk) || misaligned(Wv) || misaligned(Wo) || misaligned(k_cache) || misaligned(v_cache) ||
        misaligned(y) || (scores && misaligned(scores)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    MhaWorkspace ws(*shape, max_len, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores ? scores : ws.base.scores;
    uint8_t *mk = mask ? mask : ws.base.mask;
    // the predictor and the mask builder are the FFN's: one significance value per head
    hipError_t e = launch_predictor(shape->dtype, x_pred, 1, shape->d, shape->rank, shape->n_heads, At, Bt,
                                    ws.base.h, nullptr, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    e = launch_scores_and_mask(shape->dtype, ws.base.h, Bt, shape->rank, sc, 1, shape->n_heads, k_keep, prio_dev,
                               n_dev, drop, order, group_dev, mk, surv_idx, n_surv, s);
    if (e != hipSuccess) return HALO_ERR_HIP;
    e = launch_mha_decode(x, shape->d, shape->n_heads, Wq, Wk, Wv, Wo, k_cache, v_cache, max_len, pos, mk, y,
                          ws.mha, s);
    return e == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}

int halo_mha_forward_ahead(const halo_mha_shape *shape, const void *x, const void *Wq, const void *Wk,
                           const void *Wv, const void *Wo, void *k_cache, void *v_cache, int32_t max_len,
                           int32_t pos, const uint8_t *mask_cur, void *y, const void *x_pred_next,
                           const void *At_next, const void *Bt_next, int32_t k_keep, const int8_t *prio_dev,
                           int32_t n_dev, const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                           int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                           int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_mha_shape(shape);
    if (rc) return rc;
    if (max_len < 1 || max_len > kMhaMaxLen || pos < 0 || pos >= max_len || k_keep < 0 ||
        k_keep > shape->n_heads || n_dev < 1 || n_dev > 127)
        return HALO_ERR_ARG;
    if (!x || !Wq || !Wk || !Wv || !Wo || !k_cache || !v_cache || !mask_cur || !y || !x_pred_next || !At_next ||
        !Bt_next || !mask_next || (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (mask_next == mask_cur || y == x_pred_next) return HALO_ERR_ARG;
    if (misaligned(x) || misaligned(Wq) || misaligned(Wk) || misaligned(Wv) || misaligned(Wo) ||
        misaligned(k_cache) || misaligned(v_cache) || misaligned(y) || misaligned(x_pred_next) ||
        misaligned(At_next) || misaligned(Bt_next) || (scores_next && misaligned(scores_next)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    MhaWorkspace ws(*shape, max_len, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores_next ? scores_next : ws.base.scores;
    AheadArgs ah{x_pred_next, At_next, Bt_next, shape->rank, k_keep, n_dev, prio_dev, drop_next, ws.base.h, sc,
                 order_next, group_dev_next, mask_next, surv_idx_next, n_surv_next};
    bool fused = false;
    hipError_t e = launch_mha_decode(x, shape->d, shape->n_heads, Wq, Wk, Wv, Wo, k_cache, v_cache, max_len, pos,
                                     mask_cur, y, ws.mha, s, &ah, &fused);
    if (e != hipSuccess) return HALO_ERR_HIP;
    if (!fused) {
        e = launch_predictor(shape->dtype, x_pred_next, 1, shape->d, shape->rank, shape->n_heads, At_next, Bt_next,
                             ws.base.h, nullptr, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
        e = launch_scores_and_mask(shape->dtype, ws.base.h, Bt_next, shape->rank, sc, 1, shape->n_heads, k_keep,
                                   prio_dev, n_dev, drop_next, order_next, group_dev_next, mask_next,
                                   surv_idx_next, n_surv_next, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
    }
    return HALO_OK;
}

int halo_ffn_forward_ahead_q4(const halo_shape *shape, const void *x, int32_t T, const void *Wg_codes,
                              const void *Wg_scales, const void *Wu_codes, const void *Wu_scales,
                              const void *Wd_codes, const void *Wd_scales, const uint8_t *mask_cur, void *y,
                              const void *x_pred_next, const void *At_next, const void *Bt_next,
                              int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                              const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                              int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                              int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!q4_shape_supported(shape->d, shape->group_size)) return HALO_ERR_SHAPE;
    if (T < 0 || k_keep < 0 || k_keep > shape->n_groups || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !Wg_codes || !Wg_scales || !Wu_codes || !Wu_scales || !Wd_codes || !Wd_scales || !mask_cur ||
        !y || !x_pred_next || !At_next || !Bt_next || !mask_next || (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (mask_next == mask_cur || y == x_pred_next) return HALO_ERR_ARG;
    if (misaligned(x) || misaligned(Wg_codes) || misaligned(Wg_scales) || misaligned(Wu_codes) ||
        misaligned(Wu_scales) || misaligned(Wd_codes) || misaligned(Wd_scales) || misaligned(y) ||
        misaligned(x_pred_next) || misaligned(At_next) || misaligned(Bt_next) ||
        (scores_next && misaligned(scores_next)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws = q4_workspace(*shape, T, k_keep, workspace, ws_bytes);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores_next ? scores_next : ws.scores;
    AheadArgs ah{x_pred_next, At_next, Bt_next, shape->rank, k_keep, n_dev, prio_dev, drop_next, ws.h, sc,
                 order_next, group_dev_next, mask_next, surv_idx_next, n_surv_next};
    const Q4Weights w{(const uint32_t *)Wg_codes, (const bf16_t *)Wg_scales, (const uint32_t *)Wu_codes,
                      (const bf16_t *)Wu_scales, (const uint32_t *)Wd_codes, (const bf16_t *)Wd_scales};
    bool fused = false;
    hipError_t e = launch_ffn_q4(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size, w, mask_cur,
                                 y, ws.dec, s, shape->rank, &ah, &fused);
    if (e != hipSuccess) return HALO_ERR_HIP;
    if (!fused) {
        e = launch_predictor(shape->dtype, x_pred_next, T, shape->d, shape->rank, shape->n_groups, At_next,
                             Bt_next, ws.h, nullptr, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
        e = launch_scores_and_mask(shape->dtype, ws.h, Bt_next, shape->rank, sc, T, shape->n_groups, k_keep,
                                   prio_dev, n_dev, drop_next, order_next, group_dev_next, mask_next,
                                   surv_idx_next, n_surv_next, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
    }
    return HALO_OK;
}

int halo_ffn_forward_ahead(const halo_shape *shape, const void *x, int32_t T, const void *Wg,
                           const void *Wu, const void *Wd, const uint8_t *mask_cur, void *y,
                           const void *x_pred_next, const void *At_next, const void *Bt_next,
                           int32_t k_keep, const int8_t *prio_dev, int32_t n_dev,
                           const uint8_t *drop_next, float *scores_next, int32_t *order_next,
                           int8_t *group_dev_next, uint8_t *mask_next, int32_t *surv_idx_next,
                           int32_t *n_surv_next, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_shape(shape);
    if (rc) return rc;
    if (T < 0 || k_keep < 0 || k_keep > shape->n_groups || n_dev < 1 || n_dev > 127) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    if (!x || !Wg || !Wu || !Wd || !mask_cur || !y || !x_pred_next || !At_next || !Bt_next ||
        !mask_next || (k_keep > 0 && !prio_dev))
        return HALO_ERR_NULL;
    if (mask_next == mask_cur || y == x_pred_next) return HALO_ERR_ARG;
    if (misaligned(x) || misaligned(Wg) || misaligned(Wu) || misaligned(Wd) || misaligned(y) ||
        misaligned(x_pred_next) || misaligned(At_next) || misaligned(Bt_next) ||
        (scores_next && misaligned(scores_next)))
        return HALO_ERR_ARG;
    if (!workspace || misaligned(workspace)) return HALO_ERR_WORKSPACE;
    Workspace ws(*shape, T, k_keep, workspace);
    if (ws_bytes < ws.bytes) return HALO_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sc = scores_next ? scores_next : ws.scores;
    AheadArgs ah{x_pred_next, At_next, Bt_next, shape->rank, k_keep, n_dev, prio_dev, drop_next, ws.h, sc,
                 order_next, group_dev_next, mask_next, surv_idx_next, n_surv_next};
    bool fused = false;
    hipError_t e = launch_ffn_decode(shape->dtype, x, T, shape->d, shape->n_groups, shape->group_size, Wg,
                                     Wu, Wd, mask_cur, y, ws.dec, s, &ah, &fused);
    if (e != hipSuccess) return HALO_ERR_HIP;
    if (!fused) {
        // no path with spare workgroups for this shape: the prediction follows on the stream
        e = launch_predictor(shape->dtype, x_pred_next, T, shape->d, shape->rank, shape->n_groups, At_next,
                             Bt_next, ws.h, nullptr, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
        e = launch_scores_and_mask(shape->dtype, ws.h, Bt_next, shape->rank, sc, T, shape->n_groups, k_keep,
                                   prio_dev, n_dev, drop_next, order_next, group_dev_next, mask_next,
                                   surv_idx_next, n_surv_next, s);
        if (e != hipSuccess) return HALO_ERR_HIP;
    }
    return HALO_OK;
}

}  // extern "C"
