// Head-sparse multi-head attention for one new token (paper Sec. II-A: in the MHA one head
// and its slice of the output projection are one neuron group, the block output is the sum
// of the groups' partial results; Sec. III-B.3: every device keeps the full KV cache).
//
//   every head h     : k_h = Wk_h x, v_h = Wv_h x  -> row `pos` of the caches (storage type)
//   surviving heads  : q_h = Wq_h x,  p = softmax(q_h K_h^T / sqrt(dh)) over rows 0..pos,
//                      o_h = p V_h,   y = sum_h Wo_h o_h
//
// bf16, head dimension 128.  Four launches:
//   qkv_rows     : a matrix-vector product over the rows that are needed -- all of Wk and Wv,
//                  and the rows of Wq of surviving heads only -- streamed like the FFN's
//                  gate/up rows (one wave per row, 16-byte non-temporal loads, two rows
//                  in flight while two are reduced).
//   attn_partial : one workgroup per (surviving head, 128 cached positions): scores, a local
//                  softmax (max, sum) and the weighted sum of the values of its positions.
//   attn_combine : merges a head's partial softmaxes into o_h (bf16).
//   out-proj     : the FFN's down-projection kernel, unchanged: Wo is stored head-blocked
//                  [H][d][128] exactly like Wd, heads play the role of groups.
// Only surviving heads' query rows, cache rows and output-projection blocks are read.
#include "kernels.hpp"
#include "mask_words.hpp"

namespace halo {

constexpr int kHeadDim = 128;
constexpr int kAttnChunk = 128;      // cached positions per workgroup of attn_partial

// ---------------------------------------------------------------------------
// q / k / v rows: grid = 256 workgroups of 256 threads
// ---------------------------------------------------------------------------
// Row v of the job list: v < H*dh -> Wk row v, < 2*H*dh -> Wv row, else a Wq row of the
// (v - 2*H*dh) / dh -th surviving head.  K/V rows do not depend on the mask, so every wave
// starts on its share of them at once and meets the mask only for its query rows.
template <int NCH>
struct RowRegs {
    u32x4 a[NCH], b[NCH];            // two independent rows
};

template <int NCH>
__device__ __forceinline__ void load_two(RowRegs<NCH> &r, const bf16_t *pa, const bf16_t *pb, int lane)
{
    const u32x4 *qa = reinterpret_cast<const u32x4 *>(pa) + lane, *qb = reinterpret_cast<const u32x4 *>(pb) + lane;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        r.a[k] = __builtin_nontemporal_load(qa + k * kWave);
        r.b[k] = __builtin_nontemporal_load(qb + k * kWave);
    }
}

template <int NCH>
__device__ __forceinline__ void dot_two(const RowRegs<NCH> &r, const u32x4 (&xr)[NCH], float &ra, float &rb)
{
    float a0 = 0.0f, b0 = 0.0f;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        a0 = dot2_bf16(r.a[k].x, xr[k].x, a0);
        b0 = dot2_bf16(r.b[k].x, xr[k].x, b0);
        a0 = dot2_bf16(r.a[k].y, xr[k].y, a0);
        b0 = dot2_bf16(r.b[k].y, xr[k].y, b0);
        a0 = dot2_bf16(r.a[k].z, xr[k].z, a0);
        b0 = dot2_bf16(r.b[k].z, xr[k].z, b0);
        a0 = dot2_bf16(r.a[k].w, xr[k].w, a0);
        b0 = dot2_bf16(r.b[k].w, xr[k].w, b0);
    }
    ra = wave_sum_fast(a0);
    rb = wave_sum_fast(b0);
}

struct QkvArgs {
    const bf16_t *x, *Wq, *Wk, *Wv;
    bf16_t *k_cache, *v_cache;       // [H][max_len][128]
    float *q;                        // [n_surv][128], compact by surviving-head slot
    const uint8_t *mask;             // [H]
    int H, max_len, pos;
    // the next block's first predictor layer, in the first n_pred workgroups (0 = none)
    const bf16_t *x_next, *At_next;
    float *h_next;
    int r, n_pred;
};

// pairs of rows [p0, p1) of a job list whose row v comes from src(v) and goes to put(v, value)
template <int NCH, typename Src, typename Put>
__device__ __forceinline__ void sweep_pairs(int p0, int p1, const u32x4 (&xr)[NCH], int lane, Src src, Put put)
{
    if (p0 >= p1) return;
    RowRegs<NCH> A, B;
    load_two<NCH>(A, src(2 * p0), src(2 * p0 + 1), lane);
    int p = p0;
    while (p + 2 < p1) {
        load_two<NCH>(B, src(2 * p + 2), src(2 * p + 3), lane);
        float va, vb;
        dot_two<NCH>(A, xr, va, vb);
        put(2 * p, va);
        put(2 * p + 1, vb);
        load_two<NCH>(A, src(2 * p + 4), src(2 * p + 5), lane);
        dot_two<NCH>(B, xr, va, vb);
        put(2 * p + 2, va);
        put(2 * p + 3, vb);
        p += 2;
    }
    if (p + 1 < p1) {
        load_two<NCH>(B, src(2 * p + 2), src(2 * p + 3), lane);
        float va, vb;
        dot_two<NCH>(A, xr, va, vb);
        put(2 * p, va);
        put(2 * p + 1, vb);
        dot_two<NCH>(B, xr, va, vb);
        put(2 * p + 2, va);
        put(2 * p + 3, vb);
    } else {
        float va, vb;
        dot_two<NCH>(A, xr, va, vb);
        put(2 * p, va);
        put(2 * p + 1, vb);
    }
}

template <int NCH>
__global__ __launch_bounds__(256) void qkv_rows(QkvArgs a)
{
    constexpr int d = NCH * 512, dh = kHeadDim;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if ((int)blockIdx.x < a.n_pred) {
        // paper Sec. III-B.3, Pred beside Load/Comp, one layer ahead: h_next = ReLU(x_next A)
        const int j = blockIdx.x * 4 + wave;
        if (j < a.r) {
            const float p = dot_order64_fixed<d>(a.x_next, a.At_next + (size_t)j * d, lane);
            if (lane == 0) a.h_next[j] = p > 0.0f ? p : 0.0f;
        }
        return;
    }
    const int nw = (gridDim.x - a.n_pred) * 4, w = (blockIdx.x - a.n_pred) * 4 + wave;
    const MaskWords mw = load_mask_words(a.mask, a.H, lane);     // needed only further down
    u32x4 xr[NCH];
#pragma unroll
    for (int k = 0; k < NCH; ++k) xr[k] = *reinterpret_cast<const u32x4 *>(a.x + (k * kWave + lane) * 8);
    // keys and values of every head: 2*H*dh rows, taken in pairs
    {
        const int hd = a.H * dh;
        const long long pairs = hd;                              // 2*hd rows
        const int p0 = (int)(pairs * w / nw), p1 = (int)(pairs * (w + 1) / nw);
        auto src = [&](int v) -> const bf16_t * {
            return v < hd ? a.Wk + (size_t)v * d : a.Wv + (size_t)(v - hd) * d;
        };
        auto put = [&](int v, float val) {
            if (lane == 0) {
                const int r = v < hd ? v : v - hd;
                const int h = r / dh, e = r - h * dh;
                bf16_t *dst = (v < hd ? a.k_cache : a.v_cache) + ((size_t)h * a.max_len + a.pos) * dh + e;
                *dst = f32_to_bf16(val);
            }
        };
        sweep_pairs<NCH>(p0, p1, xr, lane, src, put);
    }
    // queries of the surviving heads: count*dh rows (an even number), compact by slot
    {
        const long long pairs = (long long)mw.count * (dh / 2);
        const int p0 = (int)(pairs * w / nw), p1 = (int)(pairs * (w + 1) / nw);
        int cur_u = -1, cur_g = 0;
        auto src = [&](int v) -> const bf16_t * {
            const int u = v / dh;
            if (u != cur_u) {
                cur_u = u;
                cur_g = nth_group(mw, u, lane);
            }
            return a.Wq + ((size_t)cur_g * dh + (v - u * dh)) * d;
        };
        auto put = [&](int v, float val) {
            if (lane == 0) a.q[v] = val;
        };
        sweep_pairs<NCH>(p0, p1, xr, lane, src, put);
    }
}

// any d that is a multiple of 8: one wave per row, one row at a time
__global__ __launch_bounds__(256) void qkv_rows_generic(QkvArgs a, int d, const int32_t *__restrict__ ulist,
                                                        const int32_t *__restrict__ meta)
{
    constexpr int dh = kHeadDim;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int hd = a.H * dh, total = 2 * hd + meta[0] * dh;
    for (int v = blockIdx.x * 4 + wave; v < total; v += gridDim.x * 4) {
        const bf16_t *src;
        if (v < hd) src = a.Wk + (size_t)v * d;
        else if (v < 2 * hd) src = a.Wv + (size_t)(v - hd) * d;
        else {
            const int r = v - 2 * hd, u = r / dh;
            src = a.Wq + ((size_t)ulist[u] * dh + (r - u * dh)) * d;
        }
        float p = 0.0f;
        for (int c = lane; c * 8 < d; c += kWave) {
            float xv[8], wv[8];
            load8(a.x + c * 8, xv);
            load8(src + c * 8, wv);
#pragma unroll
            for (int e = 0; e < 8; ++e) p = __builtin_fmaf(xv[e], wv[e], p);
        }
        p = wave_sum(p);
        if (lane == 0) {
            if (v < 2 * hd) {
                const int r = v < hd ? v : v - hd;
                const int h = r / dh, e = r - h * dh;
                (v < hd ? a.k_cache : a.v_cache)[((size_t)h * a.max_len + a.pos) * dh + e] = f32_to_bf16(p);
            } else {
                a.q[v - 2 * hd] = p;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// attention over the cache: grid (chunks, H), 256 threads
// ---------------------------------------------------------------------------
// Workgroup (c, u): surviving-head slot u (exits if u >= number of survivors), cached
// positions c*128 .. c*128+127 (rows beyond pos count as score -inf).  16 lanes share a
// cache row (16 bytes = 8 dimensions each), a wave covers 4 rows per instruction and 32 rows
// in all.  Output: part[(u*chunks + c)] = {local max, local sum, 128 weighted value sums}.
constexpr int kPartStride = kHeadDim + 2;

__global__ __launch_bounds__(256) void attn_partial(const float *__restrict__ q, const bf16_t *__restrict__ k_cache,
                                                    const bf16_t *__restrict__ v_cache,
                                                    const uint8_t *__restrict__ mask, int H, int max_len, int pos,
                                                    float *__restrict__ part)
{
    constexpr int dh = kHeadDim;
    __shared__ float s_score[kAttnChunk];
    __shared__ float s_o[4][dh];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c = blockIdx.x, u = blockIdx.y, chunks = gridDim.x;
    const MaskWords mw = load_mask_words(mask, H, lane);
    if (u >= mw.count) return;                                   // uniform
    const int h = nth_group(mw, u, lane);
    const int sub = lane >> 4, piece = (lane & 15) * 8;
    const bf16_t *K = k_cache + (size_t)h * max_len * dh, *V = v_cache + (size_t)h * max_len * dh;
    const int j0 = c * kAttnChunk + wave * 32;                   // this wave's first row
    // every load of the workgroup's 64 KiB is requested before anything is reduced
    u32x4 kv[8], vv[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        int j = j0 + it * 4 + sub;
        j = j <= pos ? j : pos;                                  // past the end: a valid duplicate, weight 0
        kv[it] = *reinterpret_cast<const u32x4 *>(K + (size_t)j * dh + piece);
        vv[it] = *reinterpret_cast<const u32x4 *>(V + (size_t)j * dh + piece);
    }
    float qf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] = q[u * dh + piece + e];
    const float scale = 0.08838834764831845f;                    // 1 / sqrt(128)
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        float kf[8], sdot = 0.0f;
        unpack8(kv[it], kf);
#pragma unroll
        for (int e = 0; e < 8; ++e) sdot = __builtin_fmaf(qf[e], kf[e], sdot);
        sdot = dpp_add<0xB1>(sdot);                              // the 16 lanes of a row
        sdot = dpp_add<0x4E>(sdot);
        sdot = dpp_add<0x141>(sdot);
        sdot = dpp_add<0x140>(sdot);
        const int j = j0 + it * 4 + sub;
        if ((lane & 15) == 0) s_score[wave * 32 + it * 4 + sub] = j <= pos ? sdot * scale : -INFINITY;
    }
    __syncthreads();
    // local softmax statistics (every wave computes them for itself from the 128 scores)
    float m = fmaxf(s_score[lane], s_score[lane + 64]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
    // the chunk's first row always exists (chunks are launched only up to pos), so m is finite
    float l = __expf(s_score[lane] - m) + __expf(s_score[lane + 64] - m);
    l = wave_sum(l);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const float p = __expf(s_score[wave * 32 + it * 4 + sub] - m);
        float vf[8];
        unpack8(vv[it], vf);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(p, vf[e], acc[e]);
    }
    // the four row slots of a wave, then the four waves
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        acc[e] += __shfl_xor(acc[e], 16, kWave);
        acc[e] += __shfl_xor(acc[e], 32, kWave);
    }
    if (lane < 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_o[wave][piece + e] = acc[e];
    }
    __syncthreads();
    float *out = part + ((size_t)u * chunks + c) * kPartStride;
    if (tid < dh) out[2 + tid] = s_o[0][tid] + s_o[1][tid] + s_o[2][tid] + s_o[3][tid];
    if (tid == 0) {
        out[0] = m;
        out[1] = l;
    }
}

// grid = H workgroups of 128 threads: o_u = sum_c e^{m_c - M} o_c / sum_c e^{m_c - M} l_c.
// Thread tid owns dimension tid of the head and chunk tid's statistics.  Everything the first 32 chunks
// need -- the thread's chunk maximum and sum, and its 32 value sums -- is requested before anything is
// waited for, so a cache of up to 4096 positions costs one memory round trip (with the maxima, the
// sums and the values fetched in turn, in batches of eight, it was six).
constexpr int kMaxChunks = 1024;     // 131072 cached positions

template <typename OT>
__global__ __launch_bounds__(128) void attn_combine(const float *__restrict__ part, const uint8_t *__restrict__ mask,
                                                    int H, int chunks, OT *__restrict__ act)
{
    constexpr int dh = kHeadDim, kBatch = 32;
    __shared__ float s_w[kMaxChunks];
    __shared__ float s_red[2][2];
    const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const MaskWords mw = load_mask_words(mask, H, lane);
    if (u >= mw.count) return;
    const float *p = part + (size_t)u * chunks * kPartStride;
    // the first batch of value sums and this thread's chunk statistics, all in flight together
    float v[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) v[i] = p[(size_t)(i < chunks ? i : chunks - 1) * kPartStride + 2 + tid];
    const int c_own = tid < chunks ? tid : chunks - 1;
    const float m_own = p[(size_t)c_own * kPartStride], l_own = p[(size_t)c_own * kPartStride + 1];
    // pass 1: maximum of the chunk maxima
    float m_loc = tid < chunks ? m_own : -INFINITY;
    for (int c = tid + 128; c < chunks; c += 128) m_loc = fmaxf(m_loc, p[(size_t)c * kPartStride]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m_loc = fmaxf(m_loc, __shfl_xor(m_loc, off, kWave));
    if (lane == 0) s_red[0][wave] = m_loc;
    __syncthreads();
    const float M = fmaxf(s_red[0][0], s_red[0][1]);
    // pass 2: chunk weights and the denominator
    float l_loc = 0.0f;
    if (tid < chunks) {
        const float w = __expf(m_own - M);
        s_w[tid] = w;
        l_loc = w * l_own;
    }
    for (int c = tid + 128; c < chunks; c += 128) {
        const float w = __expf(p[(size_t)c * kPartStride] - M);
        s_w[c] = w;
        l_loc = __builtin_fmaf(w, p[(size_t)c * kPartStride + 1], l_loc);
    }
    l_loc = wave_sum(l_loc);
    if (lane == 0) s_red[1][wave] = l_loc;
    __syncthreads();
    const float L = s_red[1][0] + s_red[1][1];
    float o = 0.0f;
#pragma unroll
    for (int i = 0; i < kBatch; ++i)
        if (i < chunks) o = __builtin_fmaf(s_w[i], v[i], o);
    for (int c0 = kBatch; c0 < chunks; c0 += kBatch) {
#pragma unroll
        for (int i = 0; i < kBatch; ++i) v[i] = p[(size_t)(c0 + i < chunks ? c0 + i : chunks - 1) * kPartStride + 2 + tid];
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
            if (c0 + i < chunks) o = __builtin_fmaf(s_w[c0 + i], v[i], o);
    }
    store_out(act + u * dh + tid, o / L);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
bool mha_shape_supported(int d, int head_dim) { return head_dim == kHeadDim && d % 8 == 0; }

hipError_t launch_mha_decode(const void *x, int d, int H, const void *Wq, const void *Wk, const void *Wv,
                             const void *Wo, void *k_cache, void *v_cache, int max_len, int pos,
                             const uint8_t *mask, void *y, const MhaScratch &ws, hipStream_t s,
                             const AheadArgs *ahead, bool *ahead_fused)
{
    if (ahead_fused) *ahead_fused = false;
    if (H > 256) return hipErrorInvalidValue;                    // the mask-word helpers cover 256 heads
    const int chunks = pos / kAttnChunk + 1;
    if (chunks > kMaxChunks) return hipErrorInvalidValue;
    const bool fast = d == 4096 || d == 5120 || d == 8192;
    const AheadArgs *ah = (fast && ahead && ahead_fused) ? ahead : nullptr;
    if (ah) *ahead_fused = true;
    const int n_pred = ah ? (ah->r + 3) / 4 : 0;
    QkvArgs qa{(const bf16_t *)x, (const bf16_t *)Wq, (const bf16_t *)Wk, (const bf16_t *)Wv, (bf16_t *)k_cache,
               (bf16_t *)v_cache, ws.q, mask, H, max_len, pos,
               ah ? (const bf16_t *)ah->x_next : nullptr, ah ? (const bf16_t *)ah->At : nullptr,
               ah ? ah->h : nullptr, ah ? ah->r : 0, n_pred};
    if (fast) {
        switch (d) {
        case 4096: launch_timed("qkv_rows", qkv_rows<8>, dim3(256 + n_pred), dim3(256), s, qa); break;
        case 5120: launch_timed("qkv_rows", qkv_rows<10>, dim3(256 + n_pred), dim3(256), s, qa); break;
        default: launch_timed("qkv_rows", qkv_rows<16>, dim3(256 + n_pred), dim3(256), s, qa); break;
        }
    } else {
        hipError_t e = launch_union(mask, 1, H, ws.dec.ulist, ws.dec.meta, s);
        if (e != hipSuccess) return e;
        launch_timed("qkv_rows_generic", qkv_rows_generic, dim3(512), dim3(256), s, qa, d,
                     (const int32_t *)ws.dec.ulist, (const int32_t *)ws.dec.meta);
    }
    attn_partial<<<dim3(chunks, H), dim3(256), 0, s>>>(ws.q, (const bf16_t *)k_cache, (const bf16_t *)v_cache, mask,
                                                       H, max_len, pos, ws.part);
    // the output projection is the FFN's down projection with heads as groups
    if (fast) {
        attn_combine<bf16_t><<<dim3(H), dim3(128), 0, s>>>(ws.part, mask, H, chunks,
                                                           reinterpret_cast<bf16_t *>(ws.dec.act));
        return launch_down_t1((const bf16_t *)Wo, d, H, mask, reinterpret_cast<const bf16_t *>(ws.dec.act),
                              (bf16_t *)y, s, ah);
    }
    attn_combine<float><<<dim3(H), dim3(128), 0, s>>>(ws.part, mask, H, chunks, ws.dec.act);
    return launch_down_generic_bf16(ws.dec.act, H * kHeadDim, d, kHeadDim, (const bf16_t *)Wo, ws.dec.ulist,
                                    ws.dec.meta, (bf16_t *)y, s);
}

}  // namespace halo
