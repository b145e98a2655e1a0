// Group-sparse SwiGLU FFN on the float ALUs (paper Sec. II-A neuron groups; merge = sum).
//
//   y[t] = sum_{g in S_t} sum_{m in g} Wd[g][:][m] * SiLU(Wg[g*gs+m].x[t]) * (Wu[g*gs+m].x[t])
//
// With one token the block is a memory-bound matrix-vector product: every weight element
// of a surviving group is read once, so the kernels are organised around streaming those
// bytes from HBM with 16-byte loads per lane and nothing else competing for bandwidth.
//   gate/up : one wave per neuron; lanes stride the row in 16-byte pieces, the two dot
//             products are reduced across the wave, lane 0 stores the activation.
//   down    : the down projection is stored group-blocked, Wd[g][j][m]; 16 lanes share one
//             output row j (256 bytes per group), a wave covers four rows and walks the
//             surviving groups, so no partial sums ever leave the workgroup.
// Groups that no token keeps are never addressed.
//
// This file holds the one-token hot path and a generic path (any T, d, group size, f32 or
// bf16) that favours simplicity; a few tokens in bf16 go to the matrix-core path instead.
#include "kernels.hpp"
#include "mask_device.hpp"
#include "mask_words.hpp"
#include "row_stream.hpp"

namespace halo {

// ---------------------------------------------------------------------------
// union of surviving groups over the tokens
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

hipError_t launch_union(const uint8_t *mask, int T, int G, int32_t *ulist, int32_t *meta, hipStream_t s)
{
    union_kernel<<<dim3(1), dim3(256), 0, s>>>(mask, T, G, ulist, meta);
    return hipGetLastError();
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
// generic down: one wave per output row j; lanes stride the group's neurons
// ---------------------------------------------------------------------------
template <typename WT, int TT>
__global__ __launch_bounds__(256) void down_generic(
    const float *__restrict__ act, int act_stride, int T, int d, int gs, const WT *__restrict__ Wd,
    const int32_t *__restrict__ ulist, const int32_t *__restrict__ meta, WT *__restrict__ y)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + wave;
    if (j >= d) return;
    const int n_u = meta[0];
    for (int t0 = 0; t0 < T; t0 += TT) {
        float acc[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc[tt] = 0.0f;
        for (int u = 0; u < n_u; ++u) {
            const WT *w = Wd + ((size_t)ulist[u] * d + j) * gs;
            for (int m = lane; m < gs; m += kWave) {
                const float wv = to_float(w[m]);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
                    if (t0 + tt < T)
                        acc[tt] = __builtin_fmaf(wv, act[(size_t)(t0 + tt) * act_stride + u * gs + m], acc[tt]);
            }
        }
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const float v = wave_sum(acc[tt]);
            if (lane == 0 && t0 + tt < T) store_out(y + (size_t)(t0 + tt) * d + j, v);
        }
    }
}

// ---------------------------------------------------------------------------
// one token, bf16, d = NCH*512, group size 128, G <= 256: the decode hot path
// ---------------------------------------------------------------------------
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
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, bf16_t *__restrict__ act,
    int vblock, int nblocks)
{
    constexpr int kGs = 128;                                       // the group size of this path
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const MaskWords mw = load_mask_words(mask, G, lane);
    const int total = mw.count * kGs;
    const int nw = nblocks * 4, w = vblock * 4 + wave;
    const int n0 = (int)((long long)total * w / nw), n1 = (int)((long long)total * (w + 1) / nw);
    if (n0 >= n1) return;
    // a run is shorter than a group (at most 256 groups over 1024 waves), so it touches at most two
    // groups; their ids are found once, and the row of a neuron is then a shift and a select (with
    // the lookup inside the loop, a hundred instructions stood between a reduction and the next loads)
    const int u_first = n0 / kGs, u_last = (n1 - 1) / kGs;
    const int g_first = nth_group(mw, u_first, lane), g_last = nth_group(mw, u_last, lane);
    auto row_of = [&](int n) -> size_t {
        const int u = n / kGs;
        return (size_t)(u == u_first ? g_first : g_last) * kGs + (n - u * kGs);
    };
    RowPair<NCH> A, B;
    load_rows<NCH>(A, Wg, Wu, row_of(n0), lane);
    u32x4 xr[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) xr[k] = *reinterpret_cast<const u32x4 *>(x + (k * kWave + lane) * 8);
    int n = n0;
    while (n + 2 < n1) {
        load_rows<NCH>(B, Wg, Wu, row_of(n + 1), lane);
        __builtin_amdgcn_sched_barrier(0);      // the requests go out before anything waits for the rows in flight
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = f32_to_bf16(va);
        load_rows<NCH>(A, Wg, Wu, row_of(n + 2), lane);
        __builtin_amdgcn_sched_barrier(0);
        const float vb = gate_up_dot<NCH>(B, xr);
        if (lane == 0) act[n + 1] = f32_to_bf16(vb);
        n += 2;
    }
    if (n + 1 < n1) {
        load_rows<NCH>(B, Wg, Wu, row_of(n + 1), lane);
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = f32_to_bf16(va);
        const float vb = gate_up_dot<NCH>(B, xr);
        if (lane == 0) act[n + 1] = f32_to_bf16(vb);
    } else {
        const float va = gate_up_dot<NCH>(A, xr);
        if (lane == 0) act[n] = f32_to_bf16(va);
    }
}

template <int NCH>
__global__ __launch_bounds__(256) void gate_up_t1(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, bf16_t *__restrict__ act)
{
    gate_up_t1_body<NCH>(x, G, gs, Wg, Wu, mask, act, blockIdx.x, gridDim.x);
}

// The same, with the first predictor layer of the NEXT block riding along (paper Sec. III-B.3,
// Pred beside Load/Comp, one layer ahead): the first n_pred workgroups each take four rows
// of At and produce h_next = ReLU(x_next A); the others do this block's gate/up work.
template <int NCH>
__global__ __launch_bounds__(256) void gate_up_pred_t1(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, bf16_t *__restrict__ act,
    const bf16_t *__restrict__ x_next, const bf16_t *__restrict__ At_next, int r,
    float *__restrict__ h_next, int n_pred)
{
    if ((int)blockIdx.x < n_pred) {
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const int j = blockIdx.x * 4 + wave;
        if (j < r) {
            const float p = dot_order64_fixed<NCH * 512>(x_next, At_next + (size_t)j * (NCH * 512), lane);
            if (lane == 0) h_next[j] = p > 0.0f ? p : 0.0f;
        }
        return;
    }
    gate_up_t1_body<NCH>(x, G, gs, Wg, Wu, mask, act, blockIdx.x - n_pred, gridDim.x - n_pred);
}

// Down projection for one token.  16 lanes share an output row (16 bytes each = the 128
// neurons of a group), a wave covers four rows, and two waves share those four rows, one
// taking the even and one the odd surviving groups.  A workgroup of 2*RQ waves owns 4*RQ
// consecutive rows, i.e. 1 KiB * RQ contiguous bytes of every surviving group's block.
// Each lane accumulates over its groups, the 16 lanes of a row are summed once at the end
// and the two halves meet in LDS, so y is written directly: no partial sums in memory, no
// second pass.  The activation arrives in bf16 and meets the weights in the packed dot.
constexpr int kDownBatch = 8;    // groups in flight per wave

template <int RQ>
struct DownShared {
    int list[256];
    float half[RQ][64];
};

template <int RQ>
__device__ __forceinline__ void down_t1_body(DownShared<RQ> &sh, int d, int G,
                                             const bf16_t *__restrict__ Wd,
                                             const uint8_t *__restrict__ mask,
                                             const bf16_t *__restrict__ act, bf16_t *__restrict__ y,
                                             int vblock)
{
    constexpr int gs = 128;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const MaskWords mw = load_mask_words(mask, G, lane);
    if (wave == 0) write_group_list(mw, lane, sh.list);
    __syncthreads();
    const int count = mw.count;
    const int rq = wave % RQ, half = wave / RQ;                     // row quad, even/odd groups
    const int row = (vblock * RQ + rq) * 4 + (lane >> 4);           // output index j
    const int piece = (lane & 15) * 8;                              // first neuron of this lane's piece
    const bf16_t *wbase = Wd + (size_t)row * gs + piece;
    const size_t gstride = (size_t)d * gs;
    float acc0 = 0.0f, acc1 = 0.0f;
    constexpr int kB = kDownBatch / 2;                             // two half batches in flight
    auto fetch = [&](u32x4 (&v)[kB], u32x4 (&a)[kB], int u0) {
#pragma unroll
        for (int q = 0; q < kB; ++q) {
            const int u = u0 + 2 * q < count ? u0 + 2 * q : (count > 0 ? count - 1 : 0);   // an in-range duplicate
            v[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(wbase + sh.list[u] * gstride));
            a[q] = *reinterpret_cast<const u32x4 *>(act + u * gs + piece);
        }
    };
    auto mac = [&](const u32x4 (&v)[kB], const u32x4 (&a)[kB], int u0) {
#pragma unroll
        for (int q = 0; q < kB; ++q) {
            if (u0 + 2 * q < count) {
                acc0 = dot2_bf16(v[q].x, a[q].x, acc0);
                acc1 = dot2_bf16(v[q].y, a[q].y, acc1);
                acc0 = dot2_bf16(v[q].z, a[q].z, acc0);
                acc1 = dot2_bf16(v[q].w, a[q].w, acc1);
            }
        }
    };
    if (count > 0) {
        u32x4 v0[kB], a0[kB], v1[kB], a1[kB];
        fetch(v0, a0, half);
        fetch(v1, a1, half + 2 * kB);
        int u0 = half;
        while (u0 + 4 * kB < count) {
            mac(v0, a0, u0);
            fetch(v0, a0, u0 + 4 * kB);
            mac(v1, a1, u0 + 2 * kB);
            fetch(v1, a1, u0 + 6 * kB);
            u0 += 4 * kB;
        }
        if (u0 < count) mac(v0, a0, u0);
        if (u0 + 2 * kB < count) mac(v1, a1, u0 + 2 * kB);
    }
    float v = acc0 + acc1;
    v = dpp_add<0xB1>(v);    // the 16 lanes of a row: quad_perm, quad_perm, half mirror, mirror
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    v = dpp_add<0x140>(v);
    if (half == 1) sh.half[rq][lane] = v;
    __syncthreads();
    if (half == 0 && (lane & 15) == 0) y[row] = f32_to_bf16(v + sh.half[rq][lane]);
}

// (Both down kernels are held to 128 vector registers: two workgroups must fit a compute unit, or the
// extra workgroup of the `_mask` form waits for a free one and the launch takes half as long again.)
template <int RQ>
__global__ __launch_bounds__(RQ * 128, 4) void down_t1(int d, int G, const bf16_t *__restrict__ Wd,
                                                    const uint8_t *__restrict__ mask,
                                                    const bf16_t *__restrict__ act,
                                                    bf16_t *__restrict__ y)
{
    __shared__ DownShared<RQ> sh;
    down_t1_body<RQ>(sh, d, G, Wd, mask, act, y, blockIdx.x);
}

// The down projection, with the second predictor layer + ranking + mask of the NEXT block in
// workgroup 0 (it is the longest dependent chain, so it is dispatched first).
template <int RQ>
__global__ __launch_bounds__(RQ * 128, 4) void down_mask_t1(int d, int G, const bf16_t *__restrict__ Wd,
                                                         const uint8_t *__restrict__ mask,
                                                         const bf16_t *__restrict__ act,
                                                         bf16_t *__restrict__ y, AheadDev nx)
{
    __shared__ DownShared<RQ> sh;
    __shared__ MaskShared msh;
    if (blockIdx.x == 0) {
        mask_scores_block<RQ * 128, bf16_t, true>(msh, threadIdx.x, nx.h, nx.Bt, nx.r, nx.scores, G, nx.K,
                                                  nx.prio_dev, nx.n_dev, nx.drop, nx.order, nx.group_dev,
                                                  nx.mask, nx.surv_idx, nx.n_surv);
        return;
    }
    down_t1_body<RQ>(sh, d, G, Wd, mask, act, y, blockIdx.x - 1);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
template <typename WT>
static hipError_t decode_generic(const WT *x, int T, int d, int G, int gs, const WT *Wg,
                                 const WT *Wu, const WT *Wd, const uint8_t *mask, WT *y,
                                 const DecodeScratch &ws, hipStream_t s)
{
    constexpr int TT = 4;
    const int ffn = G * gs;
    union_kernel<<<dim3(1), dim3(256), 0, s>>>(mask, T, G, ws.ulist, ws.meta);
    int blocks = (ffn + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    launch_timed("gate_up_generic", gate_up_generic<WT, TT>, dim3(blocks), dim3(256), s, x, T, d, G, gs,
                 Wg, Wu, mask, (const int32_t *)ws.ulist, (const int32_t *)ws.meta, ws.act, ffn);
    down_generic<WT, TT><<<dim3((d + 3) / 4), dim3(256), 0, s>>>(ws.act, ffn, T, d, gs, Wd, ws.ulist,
                                                               ws.meta, y);
    return hipGetLastError();
}

// One workgroup (four waves) per compute unit.  Measured in place: 384 or 512 workgroups, or
// dispatching the predictor's workgroups after the gate/up ones, are all slower.
constexpr int kGateUpBlocks = 256;

template <int NCH>
static hipError_t decode_t1(const bf16_t *x, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                            const bf16_t *Wd, const uint8_t *mask, bf16_t *y,
                            const DecodeScratch &ws, const AheadArgs *ah, hipStream_t s)
{
    constexpr int d = NCH * 512;
    bf16_t *act = reinterpret_cast<bf16_t *>(ws.act);
    if (!ah) {
        launch_timed("gate_up_t1", gate_up_t1<NCH>, dim3(kGateUpBlocks), dim3(256), s, x, G, gs, Wg, Wu,
                     mask, act);
    } else {
        const int n_pred = (ah->r + 3) / 4;
        launch_timed("gate_up_pred_t1", gate_up_pred_t1<NCH>, dim3(kGateUpBlocks + n_pred), dim3(256), s, x, G,
                     gs, Wg, Wu, mask, act, (const bf16_t *)ah->x_next, (const bf16_t *)ah->At, ah->r, ah->h,
                     n_pred);
    }
    return launch_down_t1(Wd, d, G, mask, act, y, s, ah);
}

// Row lengths of the one-token path: d = 1024 k, k = 2..8, and 5120 (LLaMA-family hidden sizes).
bool t1_shape_supported(int d)
{
    return d == 5120 || (d % 1024 == 0 && d >= 2048 && d <= 8192);
}

hipError_t launch_down_t1(const bf16_t *Wd, int d, int G, const uint8_t *mask, const bf16_t *act, bf16_t *y,
                          hipStream_t s, const AheadArgs *ahead)
{
    const AheadDev nx = ahead ? ahead_dev(*ahead) : AheadDev{};
#define HALO_DOWN_CASE(D)                                                                                  \
    case D:                                                                                                \
        if (ahead)                                                                                         \
            down_mask_t1<D / 1024><<<dim3(257), dim3(D / 1024 * 128), 0, s>>>(d, G, Wd, mask, act, y, nx); \
        else                                                                                               \
            down_t1<D / 1024><<<dim3(256), dim3(D / 1024 * 128), 0, s>>>(d, G, Wd, mask, act, y);          \
        break;
    switch (d) {
        HALO_DOWN_CASE(2048)
        HALO_DOWN_CASE(3072)
        HALO_DOWN_CASE(4096)
        HALO_DOWN_CASE(5120)
        HALO_DOWN_CASE(6144)
        HALO_DOWN_CASE(7168)
        HALO_DOWN_CASE(8192)
    default: return hipErrorInvalidValue;
    }
#undef HALO_DOWN_CASE
    return hipGetLastError();
}

hipError_t launch_down_generic_bf16(const float *act, int act_stride, int d, int gs, const bf16_t *Wd,
                                    const int32_t *ulist, const int32_t *meta, bf16_t *y, hipStream_t s)
{
    down_generic<bf16_t, 4><<<dim3((d + 3) / 4), dim3(256), 0, s>>>(act, act_stride, 1, d, gs, Wd, ulist, meta, y);
    return hipGetLastError();
}

// ahead != nullptr asks for the next block's prediction to ride along with this block's
// kernels.  The one-token path and the few-token paths (up to 16 tokens, up to 256 groups) can do
// that; *ahead_fused tells the caller whether it happened (if not, the caller enqueues the
// prediction itself).
hipError_t launch_ffn_decode(int dtype, const void *x, int T, int d, int G, int gs, const void *Wg,
                             const void *Wu, const void *Wd, const uint8_t *mask, void *y,
                             const DecodeScratch &ws, hipStream_t s, const AheadArgs *ahead,
                             bool *ahead_fused)
{
    if (ahead_fused) *ahead_fused = false;
    if (dtype == 0)
        return decode_generic<float>((const float *)x, T, d, G, gs, (const float *)Wg, (const float *)Wu,
                                     (const float *)Wd, mask, (float *)y, ws, s);
    const bf16_t *bx = (const bf16_t *)x, *bg = (const bf16_t *)Wg, *bu = (const bf16_t *)Wu,
                 *bd = (const bf16_t *)Wd;
    if (T == 1 && G <= 256 && gs == 128 && t1_shape_supported(d)) {
        const AheadArgs *ah = (ahead && ahead_fused) ? ahead : nullptr;
        if (ah) *ahead_fused = true;
        switch (d) {
        case 2048: return decode_t1<4>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 3072: return decode_t1<6>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 4096: return decode_t1<8>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 5120: return decode_t1<10>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 6144: return decode_t1<12>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        case 7168: return decode_t1<14>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        default: return decode_t1<16>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, ah, s);
        }
    }
    if (mfma_path_supported(T, d, gs))
        return launch_ffn_mfma(bx, T, d, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s, ahead, ahead_fused);
    if (prefill_path_supported(T, d, gs))
        return launch_ffn_prefill(bx, T, d, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
    return decode_generic<bf16_t>(bx, T, d, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
}

}  // namespace halo
