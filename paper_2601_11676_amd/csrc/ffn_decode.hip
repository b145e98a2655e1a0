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
//             subset of the surviving neurons; partial column sums of all subsets are
//             added in a fixed order (deterministic output, no float atomics).
// Groups that no token keeps are never addressed.
#include "kernels.hpp"

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

template <typename WT>
__global__ __launch_bounds__(256) void finalize_generic(const float *__restrict__ partial,
                                                        int n_split, long long td,
                                                        WT *__restrict__ y)
{
    const long long k = (long long)blockIdx.x * 256 + threadIdx.x;
    if (k >= td) return;
    float v = 0.0f;
    for (int i = 0; i < n_split; ++i) v += partial[(size_t)i * td + k];
    store_out(y + k, v);
}

// ---------------------------------------------------------------------------
// one token, bf16, d = NCH*512: the decode hot path
// ---------------------------------------------------------------------------
// Surviving groups of the single token, compacted in ascending order into LDS.
__device__ __forceinline__ int compact_mask_t1(const uint8_t *__restrict__ mask, int G,
                                               int *s_list, int *s_n)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave == 0) {
        int base = 0;
        for (int g0 = 0; g0 < G; g0 += kWave) {
            const int g = g0 + lane;
            const bool m = g < G && mask[g] != 0;
            const unsigned long long b = __ballot(m);
            if (m) s_list[base + __popcll(b & ((1ull << lane) - 1ull))] = g;
            base += __popcll(b);
        }
        if (lane == 0) *s_n = base;
    }
    __syncthreads();
    return *s_n;
}

template <int NCH>
__global__ __launch_bounds__(256) void gate_up_t1(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, float *__restrict__ act,
    int32_t *__restrict__ counters, int n_counters)
{
    __shared__ int s_list[1024];
    __shared__ int s_n;
    constexpr int d = NCH * 512;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (blockIdx.x == 0)
        for (int k = threadIdx.x; k < n_counters; k += 256) counters[k] = 0;
    float xr[NCH][8];
#pragma unroll
    for (int k = 0; k < NCH; ++k) load8(x + (k * kWave + lane) * 8, xr[k]);
    const int total = compact_mask_t1(mask, G, s_list, &s_n) * gs;
    const int nwaves = gridDim.x * 4;
    for (int n = blockIdx.x * 4 + wave; n < total; n += nwaves) {
        const int u = n / gs, m = n - u * gs;
        const size_t row = (size_t)s_list[u] * gs + m;
        const u32x4 *pg = reinterpret_cast<const u32x4 *>(Wg + row * d) + lane;
        const u32x4 *pu = reinterpret_cast<const u32x4 *>(Wu + row * d) + lane;
        u32x4 vg[NCH], vu[NCH];
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            vg[k] = __builtin_nontemporal_load(pg + k * kWave);
            vu[k] = __builtin_nontemporal_load(pu + k * kWave);
        }
        float ag = 0.0f, au = 0.0f;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            float a[8], b[8];
            unpack8(vg[k], a);
            unpack8(vu[k], b);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ag = __builtin_fmaf(a[e], xr[k][e], ag);
                au = __builtin_fmaf(b[e], xr[k][e], au);
            }
        }
        ag = wave_sum(ag);
        au = wave_sum(au);
        if (lane == 0) act[n] = silu_mul(ag, au);
    }
}

// grid (d/512, n_split).  The last workgroup to finish a column slice adds the
// n_split partial sums in index order and writes y.
constexpr int kDownUnroll = 4;

__global__ __launch_bounds__(256) void down_t1(
    int d, int G, int gs, const bf16_t *__restrict__ WdT, const uint8_t *__restrict__ mask,
    const float *__restrict__ act, float *__restrict__ partial, int32_t *__restrict__ counters,
    bf16_t *__restrict__ y)
{
    __shared__ int s_list[1024];
    __shared__ int s_n;
    __shared__ float red[4][512];
    __shared__ int s_ticket;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n_split = gridDim.y, i = blockIdx.y, cb = blockIdx.x;
    const int col0 = cb * 512 + lane * 8;
    const int total = compact_mask_t1(mask, G, s_list, &s_n) * gs;
    const int per = (total + n_split - 1) / n_split;
    const int n0 = i * per, n1 = min(total, n0 + per);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    int n = n0 + wave;
    for (; n + 4 * (kDownUnroll - 1) < n1; n += 4 * kDownUnroll) {
        u32x4 v[kDownUnroll];
        float a[kDownUnroll];
#pragma unroll
        for (int q = 0; q < kDownUnroll; ++q) {
            const int nn = n + 4 * q;
            const int u = nn / gs, m = nn - u * gs;
            const size_t row = (size_t)s_list[u] * gs + m;
            v[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(WdT + row * d + col0));
            a[q] = act[nn];
        }
#pragma unroll
        for (int q = 0; q < kDownUnroll; ++q) {
            float w[8];
            unpack8(v[q], w);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(a[q], w[e], acc[e]);
        }
    }
    for (; n < n1; n += 4) {
        const int u = n / gs, m = n - u * gs;
        const size_t row = (size_t)s_list[u] * gs + m;
        float w[8];
        load8(WdT + row * d + col0, w);
        const float a = act[n];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(a, w[e], acc[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][lane * 8 + e] = acc[e];
    __syncthreads();
    for (int c = threadIdx.x; c < 512; c += 256)
        partial[(size_t)i * d + cb * 512 + c] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&counters[cb], 1);
    __syncthreads();
    if (s_ticket != n_split - 1) return;
    __threadfence();
    for (int c = threadIdx.x; c < 512; c += 256) {
        float v = 0.0f;
        for (int k = 0; k < n_split; ++k)
            v += __hip_atomic_load(partial + (size_t)k * d + cb * 512 + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        y[cb * 512 + c] = f32_to_bf16(v);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int decode_n_split(int T, int d)
{
    const int ncb = (d + 511) / 512;
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
    gate_up_generic<WT, TT><<<dim3(blocks), dim3(256), 0, s>>>(x, T, d, G, gs, Wg, Wu, mask, ws.ulist,
                                                             ws.meta, ws.act, ffn);
    const int ncb = (d + 511) / 512;
    down_generic<WT, TT><<<dim3(ncb, ws.n_split), dim3(256), 0, s>>>(ws.act, ffn, T, d, gs, WdT,
                                                                   ws.ulist, ws.meta, ws.partial);
    const long long td = (long long)T * d;
    finalize_generic<WT><<<dim3((unsigned)((td + 255) / 256)), dim3(256), 0, s>>>(ws.partial, ws.n_split, td, y);
    return hipGetLastError();
}

template <int NCH>
static hipError_t decode_t1(const bf16_t *x, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                            const bf16_t *WdT, const uint8_t *mask, bf16_t *y,
                            const DecodeScratch &ws, hipStream_t s)
{
    constexpr int d = NCH * 512;
    gate_up_t1<NCH><<<dim3(512), dim3(256), 0, s>>>(x, G, gs, Wg, Wu, mask, ws.act, ws.meta + 16, NCH);
    down_t1<<<dim3(NCH, ws.n_split), dim3(256), 0, s>>>(d, G, gs, WdT, mask, ws.act, ws.partial,
                                                       ws.meta + 16, y);
    return hipGetLastError();
}

hipError_t launch_ffn_decode(int dtype, const void *x, int T, int d, int G, int gs, const void *Wg,
                             const void *Wu, const void *WdT, const uint8_t *mask, void *y,
                             const DecodeScratch &ws, hipStream_t s)
{
    if (dtype == 0)
        return decode_generic<float>((const float *)x, T, d, G, gs, (const float *)Wg, (const float *)Wu,
                                     (const float *)WdT, mask, (float *)y, ws, s);
    const bf16_t *bx = (const bf16_t *)x, *bg = (const bf16_t *)Wg, *bu = (const bf16_t *)Wu,
                 *bd = (const bf16_t *)WdT;
    if (T == 1) {
        switch (d) {
        case 4096: return decode_t1<8>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
        case 5120: return decode_t1<10>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
        case 8192: return decode_t1<16>(bx, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
        default: break;
        }
    }
    return decode_generic<bf16_t>(bx, T, d, G, gs, bg, bu, bd, mask, (bf16_t *)y, ws, s);
}

}  // namespace halo
