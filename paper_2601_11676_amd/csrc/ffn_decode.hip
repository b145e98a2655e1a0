// Group-sparse SwiGLU FFN on the float ALUs (paper Sec. II-A neuron groups; merge = sum).
//
//   y[t] = sum_{g in S_t} sum_{m in g} WdT[m][:] * SiLU(Wg[m].x[t]) * (Wu[m].x[t])
//
// With one or a few tokens the block is a memory-bound matrix-vector product: every
// weight element of a surviving group is read once and used T times, so the kernels
// are organised around streaming those rows from HBM with 16-byte loads per lane and
// nothing else competing for bandwidth.  Two phases:
//   gate/up : one wave per neuron; lanes stride the row in 16-byte pieces, the two
//             dot products are reduced across the wave, lane 0 stores the activation.
//   down    : a workgroup owns a 512-column slice of d (8 columns per lane) and a
//             subset of the surviving neurons; a small kernel then adds the subsets'
//             partial column sums in a fixed order (deterministic, no float atomics).
// Groups that no token keeps are never addressed.
#include "kernels.hpp"
#include "mask_device.hpp"

namespace halo {

// ---------------------------------------------------------------------------
// union of surviving groups over the tokens (generic path)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void union_kernel(const uint8_t *__restrict__ mask, int T, int G,
                                                    int32_t *__restrict__ ulist,
                                                    int32_t *__restrict__ meta)
{
    __shared__ uint8_t any[1024];
    const int tid = threadIdx.x;
    for (int g = tid; g < G; g += 256) {
        uint8_t a = 0;
        for (int t = 0; t < T; ++t) a |= mask[(size_t)t * G + g];
        any[g] = a ? 1 : 0;
    }
    __syncthreads();
    for (int g = tid; g < G; g += 256) {
        if (!any[g]) continue;
        int c = 0;
        for (int h = 0; h < g; ++h) c += any[h];
        ulist[c] = g;
    }
    if (tid == 0) {
        int c = 0;
        for (int h = 0; h < G; ++h) c += any[h];
        meta[0] = c;
    }
}

// ---------------------------------------------------------------------------
// generic gate/up: any d (multiple of 8), any T, TT tokens per pass over a row
// ---------------------------------------------------------------------------
template <typename WT, int TT>
__global__ __launch_bounds__(256) void gate_up_generic(
    const WT *__restrict__ x, int T, int d, int G, int gs, const WT *__restrict__ Wg,
    const WT *__restrict__ Wu, const uint8_t *__restrict__ mask, const int32_t *__restrict__ ulist,
    const int32_t *__restrict__ meta, float *__restrict__ act, int act_stride)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int total = meta[0] * gs;
    const int nwaves = gridDim.x * 4;
    for (int n = blockIdx.x * 4 + wave; n < total; n += nwaves) {
        const int u = n / gs, m = n - u * gs;
        const int g = ulist[u];
        const size_t row = (size_t)g * gs + m;
        const WT *wg = Wg + row * d, *wu = Wu + row * d;
        for (int t0 = 0; t0 < T; t0 += TT) {
            float ag[TT], au[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) ag[tt] = au[tt] = 0.0f;
            for (int c = lane; c * 8 < d; c += kWave) {
                float a[8], b[8];
                load8(wg + c * 8, a);
                load8(wu + c * 8, b);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    if (t0 + tt < T) {
                        float xv[8];
                        load8(x + (size_t)(t0 + tt) * d + c * 8, xv);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            ag[tt] = __builtin_fmaf(a[e], xv[e], ag[tt]);
                            au[tt] = __builtin_fmaf(b[e], xv[e], au[tt]);
                        }
                    }
                }
            }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const float sg = wave_sum(ag[tt]), su = wave_sum(au[tt]);
                const int t = t0 + tt;
                if (lane == 0 && t < T)
                    act[(size_t)t * act_stride + n] = mask[(size_t)t * G + g] ? silu_mul(sg, su) : 0.0f;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// generic down: grid (ceil(d/512), n_split)
// ---------------------------------------------------------------------------
template <typename WT, int TT>
__global__ __launch_bounds__(256) void down_generic(
    const float *__restrict__ act, int act_stride, int T, int d, int gs,
    const WT *__restrict__ WdT, const int32_t *__restrict__ ulist, const int32_t *__restrict__ meta,
    float *__restrict__ partial)
{
    __shared__ float red[4][TT][512];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_split = gridDim.y, i = blockIdx.y;
    const int col0 = blockIdx.x * 512 + lane * 8;
    const bool col_ok = col0 < d;
    const int total = meta[0] * gs;
    const int per = (total + n_split - 1) / n_split;
    const int n0 = i * per, n1 = min(total, n0 + per);
    for (int t0 = 0; t0 < T; t0 += TT) {
        float acc[TT][8];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[tt][e] = 0.0f;
        if (col_ok) {
            for (int n = n0 + wave; n < n1; n += 4) {
                const int u = n / gs, m = n - u * gs;
                const size_t row = (size_t)ulist[u] * gs + m;
                float w[8];
                load8(WdT + row * d + col0, w);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    if (t0 + tt < T) {
                        const float a = act[(size_t)(t0 + tt) * act_stride + n];
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[tt][e] = __builtin_fmaf(a, w[e], acc[tt][e]);
                    }
                }
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int e = 0; e < 8; ++e) red[wave][tt][lane * 8 + e] = acc[tt][e];
        __syncthreads();
        for (int k = threadIdx.x; k < TT * 512; k += 256) {
            const int tt = k / 512, c = k - tt * 512;
            const int t = t0 + tt, col = blockIdx.x * 512 + c;
            if (t < T && col < d) {
                const float v = ((red[0][tt][c] + red[1][tt][c]) + red[2][tt][c]) + red[3][tt][c];
                partial[((size_t)i * T + t) * d + col] = v;
            }
        }
        __syncthreads();
    }
}

// y[k] = sum_i partial[i][k] (k over T*d).  64 outputs per workgroup; four quarter-sums over
// i = q, q+4, ... are formed concurrently and combined in a fixed order.
template <typename WT>
__global__ __launch_bounds__(256) void finalize_generic(const float *__restrict__ partial,
                                                        int n_split, long long td,
                                                        WT *__restrict__ y)
{
    __shared__ float red[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const long long k = (long long)blockIdx.x * 64 + c;
    float v = 0.0f;
    if (k < td) {
#pragma unroll 8
        for (int i = q; i < n_split; i += 4) v += partial[(size_t)i * td + k];
    }
    red[q][c] = v;
    __syncthreads();
    if (q == 0 && k < td) store_out(y + k, ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c]);
}

// ---------------------------------------------------------------------------
// one token, bf16, d = NCH*512, G <= 256: the decode hot path
// ---------------------------------------------------------------------------
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

template <int NCH>
struct RowPair {
    u32x4 g[NCH], u[NCH];
};

template <int NCH>
__device__ __forceinline__ void load_rows(RowPair<NCH> &r, const bf16_t *__restrict__ Wg,
                                          const bf16_t *__restrict__ Wu, size_t row, int lane)
{
    constexpr int d = NCH * 512;
    const u32x4 *pg = reinterpret_cast<const u32x4 *>(Wg + row * d) + lane;
    const u32x4 *pu = reinterpret_cast<const u32x4 *>(Wu + row * d) + lane;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        r.g[k] = __builtin_nontemporal_load(pg + k * kWave);
        r.u[k] = __builtin_nontemporal_load(pu + k * kWave);
    }
}

// x stays packed (two bf16 per register); products go through the packed dot instruction
template <int NCH>
__device__ __forceinline__ float gate_up_dot(const RowPair<NCH> &r, const u32x4 (&xr)[NCH])
{
    float ag = 0.0f, au = 0.0f;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        ag = dot2_bf16(r.g[k].x, xr[k].x, ag);
        au = dot2_bf16(r.u[k].x, xr[k].x, au);
        ag = dot2_bf16(r.g[k].y, xr[k].y, ag);
        au = dot2_bf16(r.u[k].y, xr[k].y, au);
        ag = dot2_bf16(r.g[k].z, xr[k].z, ag);
        au = dot2_bf16(r.u[k].z, xr[k].z, au);
        ag = dot2_bf16(r.g[k].w, xr[k].w, ag);
        au = dot2_bf16(r.u[k].w, xr[k].w, au);
    }
    return silu_mul(wave_sum_fast(ag), wave_sum_fast(au));
}

// One wave per neuron at a time; each wave owns a contiguous run of the surviving neurons
// (runs differ by at most one neuron) and keeps the next neuron's two rows in flight while
// it reduces the current one.  The steady-state loop has no branch between a load batch
// and the reduction that precedes it, so the wait counters can leave that batch in flight.
// vblock / nblocks: this workgroup's index among the workgroups doing this job.
template <int NCH>
__device__ __forceinline__ void gate_up_t1_body(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, float *__restrict__ act,
    int vblock, int nblocks)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const MaskWords mw = load_mask_words(mask, G, lane);
    const long long total = (long long)mw.count * gs;
    const int nw = nblocks * 4, w = vblock * 4 + wave;
    const int n0 = (int)(total * w / nw), n1 = (int)(total * (w + 1) / nw);
    if (n0 >= n1) return;
    int cur_u = n0 / gs;
    int cur_g = nth_group(mw, cur_u, lane);
    auto row_of = [&](int n) -> size_t {
        const int u = n / gs;
        if (u != cur_u) {
            cur_u = u;
            cur_g = nth_group(mw, u, lane);
        }
        return (size_t)cur_g * gs + (n - u * gs);
    };
    RowPair<NCH> A, B;
    load_rows<NCH>(A, Wg, Wu, row_of(n0), lane);
    u32x4 xr[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) xr[k] = *reinterpret_cast<const u32x4 *>(x + (k * kWave + lane) * 8);
    int n = n0;
    while (n + 2 < n1) {
        load_rows<NCH>(B, Wg, Wu, row_of(n + 1), lane);
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = va;
        load_rows<NCH>(A, Wg, Wu, row_of(n + 2), lane);
        const float vb = gate_up_dot<NCH>(B, xr);
        if (lane == 0) act[n + 1] = vb;
        n += 2;
    }
    if (n + 1 < n1) {
        load_rows<NCH>(B, Wg, Wu, row_of(n + 1), lane);
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = va;
        const float vb = gate_up_dot<NCH>(B, xr);
        if (lane == 0) act[n + 1] = vb;
    } else {
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = va;
    }
}

// arrival counters of the down-projection kernel that follows on the stream
template <int NCH>
__device__ __forceinline__ void reset_counters(int32_t *counters)
{
    if (threadIdx.x < NCH)
        __hip_atomic_store(counters + threadIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NCH>
__global__ __launch_bounds__(256) void gate_up_t1(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, float *__restrict__ act,
    int32_t *__restrict__ counters)
{
    if (blockIdx.x == 0) reset_counters<NCH>(counters);
    gate_up_t1_body<NCH>(x, G, gs, Wg, Wu, mask, act, blockIdx.x, gridDim.x);
}

// The same, with the first predictor layer of the NEXT block riding along (paper Sec. III-B.3,
// Pred beside Load/Comp, one layer ahead): the first n_pred workgroups each take four rows
// of At and produce h_next = ReLU(x_next A); the others do this block's gate/up work.
template <int NCH>
__global__ __launch_bounds__(256) void gate_up_pred_t1(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, float *__restrict__ act,
    int32_t *__restrict__ counters, const bf16_t *__restrict__ x_next,
    const bf16_t *__restrict__ At_next, int r, float *__restrict__ h_next, int n_pred)
{
    if ((int)blockIdx.x < n_pred) {
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const int j = blockIdx.x * 4 + wave;
        if (j < r) {
            const float p = dot_order64(x_next, At_next + (size_t)j * (NCH * 512), NCH * 512, lane);
            if (lane == 0) h_next[j] = p > 0.0f ? p : 0.0f;
        }
        return;
    }
    const int vblock = blockIdx.x - n_pred;
    if (vblock == 0) reset_counters<NCH>(counters);
    gate_up_t1_body<NCH>(x, G, gs, Wg, Wu, mask, act, vblock, gridDim.x - n_pred);
}

// grid (d/512, n_split): partial[i][:] = sum over neuron subset i of act[n] * WdT[row(n)][:].
// A workgroup owns 512 columns (8 per lane); its eight waves interleave the subset's rows,
// eight rows in flight per wave.  The workgroup that arrives last at a column slice adds
// the n_split partial sums in index order (so the result does not depend on arrival order)
// and writes y.  Partials and the arrival counter are exchanged with device-scope atomic
// loads and stores, which are coherent across the chip's L2 slices without a cache-wide
// write-back; no workgroup ever waits for another.
constexpr int kDownUnroll = 8;
constexpr int kDownWaves = 8;

struct DownShared {
    int list[256];
    float red[kDownWaves][512];
    int ticket;
};

__device__ __forceinline__ void down_t1_body(
    DownShared &sh, int d, int G, int gs, const bf16_t *__restrict__ WdT,
    const uint8_t *__restrict__ mask, const float *__restrict__ act, float *partial,
    int32_t *counters, bf16_t *__restrict__ y, int cb, int i, int n_split)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int col0 = cb * 512 + lane * 8;
    const MaskWords mw = load_mask_words(mask, G, lane);
    if (wave == 0) {
        int base = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if ((mw.w[k] >> lane) & 1ull)
                sh.list[base + __popcll(mw.w[k] & ((1ull << lane) - 1ull))] = k * kWave + lane;
            base += __popcll(mw.w[k]);
        }
    }
    __syncthreads();
    const long long total = (long long)mw.count * gs;
    const int n0 = (int)(total * i / n_split), n1 = (int)(total * (i + 1) / n_split);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int n = n0 + wave; n < n1; n += kDownWaves * kDownUnroll) {
        u32x4 v[kDownUnroll];
        float a[kDownUnroll];
#pragma unroll
        for (int q = 0; q < kDownUnroll; ++q) {
            int nn = n + kDownWaves * q;
            const bool ok = nn < n1;
            nn = ok ? nn : n;        // past the end: reload an in-range row with weight 0
            const int u = nn / gs, m = nn - u * gs;
            const size_t row = (size_t)sh.list[u] * gs + m;
            v[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(WdT + row * d + col0));
            a[q] = ok ? act[nn] : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < kDownUnroll; ++q) {
            float w[8];
            unpack8(v[q], w);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(a[q], w[e], acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) sh.red[wave][lane * 8 + e] = acc[e];
    __syncthreads();
    const int c = threadIdx.x;     // 512 threads, 512 columns
    {
        float sum = 0.0f;
#pragma unroll
        for (int q = 0; q < kDownWaves; ++q) sum += sh.red[q][c];
        __hip_atomic_store(partial + (size_t)i * d + cb * 512 + c, sum, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();               // waits for this workgroup's stores before it takes a ticket
    if (threadIdx.x == 0)
        sh.ticket = __hip_atomic_fetch_add(counters + cb, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sh.ticket != n_split - 1) return;
    float v = 0.0f;
#pragma unroll 8
    for (int k = 0; k < n_split; ++k)
        v += __hip_atomic_load(partial + (size_t)k * d + cb * 512 + c, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    y[cb * 512 + c] = f32_to_bf16(v);
    if (threadIdx.x == 0)
        __hip_atomic_store(counters + cb, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(kDownWaves * 64) void down_t1(
    int d, int G, int gs, const bf16_t *__restrict__ WdT, const uint8_t *__restrict__ mask,
    const float *__restrict__ act, float *partial, int32_t *counters, bf16_t *__restrict__ y)
{
    __shared__ DownShared sh;
    down_t1_body(sh, d, G, gs, WdT, mask, act, partial, counters, y, blockIdx.x, blockIdx.y, gridDim.y);
}

// Arguments of the prediction for the next block that rides along with this block's kernels.
struct AheadDev {
    const float *h;          // [r] first-layer output, written by gate_up_pred_t1
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

// The down projection, with the second predictor layer + ranking + mask of the NEXT block in
// workgroup 0 (it is the longest dependent chain, so it is dispatched first).  1-D grid:
// block 0 = mask, block 1 + cb + ncb * i = down-projection workgroup (cb, i).
__global__ __launch_bounds__(kDownWaves * 64) void down_mask_t1(
    int d, int G, int gs, const bf16_t *__restrict__ WdT, const uint8_t *__restrict__ mask,
    const float *__restrict__ act, float *partial, int32_t *counters, bf16_t *__restrict__ y,
    int ncb, int n_split, AheadDev nx)
{
    __shared__ DownShared sh;
    __shared__ MaskShared msh;
    if (blockIdx.x == 0) {
        mask_scores_block<kDownWaves * 64, bf16_t, true>(msh, threadIdx.x, nx.h, nx.Bt, nx.r, nx.scores, G,
                                                         nx.K, nx.prio_dev, nx.n_dev, nx.drop, nx.order,
                                                         nx.group_dev, nx.mask, nx.surv_idx, nx.n_surv);
        return;
    }
    const int flat = blockIdx.x - 1;
    down_t1_body(sh, d, G, gs, WdT, mask, act, partial, counters, y, flat % ncb, flat / ncb, n_split);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int decode_n_split(int T, int d)
{
    const int ncb = (d + 511) / 512;
    if (T == 1) return 256 / ncb > 0 ? 256 / ncb : 1;   // one workgroup per compute unit
    int n = 1024 / ncb;
    if (n > 64) n = 64;
    while (n > 1 && (long long)n * T > 1024) n /= 2;   // bound the partial-sum buffer
    return n < 1 ? 1 : n;
}

template <typename WT>
static hipError_t decode_generic(const WT *x, int T, int d, int G, int gs, const WT *Wg,
                                 const WT *Wu, const WT *WdT, const uint8_t *mask, WT *y,
                                 const DecodeScratch &ws, hipStream_t s)
{
    constexpr int TT = 4;
    const int ffn = G * gs;
    union_kernel<<<dim3(1), dim3(256), 0, s>>>(mask, T, G, ws.ulist, ws.meta);
    int blocks = (ffn + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    launch_timed("gate_up_generic", gate_up_generic<WT, TT>, dim3(blocks), dim3(256), s, x, T, d, G, gs,
                 Wg, Wu, mask, (const int32_t *)ws.ulist, (const int32_t *)ws.meta, ws.act, ffn);
    const int ncb = (d + 511) / 512;
    down_generic<WT, TT><<<dim3(ncb, ws.n_split), dim3(256), 0, s>>>(ws.act, ffn, T, d, gs, WdT,
                                                                   ws.ulist, ws.meta, ws.partial);
    const long long td = (long long)T * d;
    finalize_generic<WT><<<dim3((unsigned)((td + 63) / 64)), dim3(256), 0, s>>>(ws.partial, ws.n_split, td, y);
    return hipGetLastError();
}

constexpr int kGateUpBlocks = 256;   // one workgroup (four waves) per compute unit

template <int NCH>
static hipError_t decode_t1(const bf16_t *x, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                            const bf16_t *WdT, const uint8_t *mask, bf16_t *y,
                            const DecodeScratch &ws, const AheadArgs *ah, hipStream_t s)
{
    constexpr int d = NCH * 512;
    int32_t *counters = ws.meta + 16;
    if (!ah) {
        launch_timed("gate_up_t1", gate_up_t1<NCH>, dim3(kGateUpBlocks), dim3(256), s, x, G, gs, Wg, Wu,
                     mask, ws.act, counters);
        down_t1<<<dim3(NCH, ws.n_split), dim3(kDownWaves * 64), 0, s>>>(d, G, gs, WdT, mask, ws.act,
                                                                      ws.partial, counters, y);
        return hipGetLastError();
    }
    const int n_pred = (ah->r + 3) / 4;
    launch_timed("gate_up_pred_t1", gate_up_pred_t1<NCH>, dim3(kGateUpBlocks + n_pred), dim3(256), s, x, G,
                 gs, Wg, Wu, mask, ws.act, counters, (const bf16_t *)ah->x_next, (const bf16_t *)ah->At,
                 ah->r, ah->h, n_pred);
    AheadDev nx{ah->h, (const bf16_t *)ah->Bt, ah->r, ah->K, ah->n_dev, ah->prio_dev, ah->drop,
                ah->scores, ah->order, ah->group_dev, ah->mask, ah->surv_idx, ah->n_surv};
    down_mask_t1<<<dim3(1 + NCH * ws.n_split), dim3(kDownWaves * 64), 0, s>>>(
        d, G, gs, WdT, mask, ws.act, ws.partial, counters, y, NCH, ws.n_split, nx);
    return hipGetLastError();
}

// ahead != nullptr asks for the next block's prediction to ride along with this block's
// kernels.  Only the one-token path can do that; *ahead_fused tells the caller whether it did
// (if not, the caller enqueues the prediction itself).
hipError_t launch_ffn_decode(int dtype, const void *x, int T, int d, int G, int gs, const void *Wg,
                             const void *Wu, const void *WdT, const uint8_t *mask, void *y,
                             const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead,
                             bool *ahead_fused)
{
    if (ahead_fused) *ahead_fused = false;
    if (dtype == 0)
        return decode_generic<float>((const float *)x, T, d, G, gs, (const float *)Wg, (const float *)Wu,
                                     (const float *)WdT, mask, (float *)y, ws, s);
    const bf16_t *bx = (const bf16_t *)x, *bg = (const bf16_t *)Wg, *bu = (const bf16_t *)Wu,
                 *bd = (const bf16_t *)WdT;
    if (T == 1 && G <= 256 && (d == 4096 || d == 5120 || d == 8192)) {
        const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
        if (ah) *ahead_fused = true;
        switch (d) {
        case 4096: return decode_t1<8>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 5120: return decode_t1<10>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        default: return decode_t1<16>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        }
    }
    return decode_generic<bf16_t>(bx, T, d, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
}

}  // namespace halo
