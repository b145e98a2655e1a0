// Gate/up projection for a few tokens (2..4) on the float ALUs, bf16.
//
// With a handful of tokens the block is still bound by streaming the union of the tokens'
// surviving groups from HBM: 2*T multiply-adds per weight element fit beside the memory time of
// that element as long as T is small.  So the kernel is the one-token kernel with more columns:
// one wave per neuron, the neuron's gate and up rows fetched with 16-byte non-temporal loads
// (1 KiB of consecutive bytes per instruction, no re-shaping), the next neuron's rows in flight
// while the current one is reduced, and every weight register used T times against the token
// rows of x, which live in LDS for the whole kernel.  (The matrix-core form of this kernel
// re-shapes every weight tile through LDS and keeps fewer bytes in flight per row; it reached
// 3.5 TB/s on a 63-group union of the 13B shape and 5.8 TB/s on the 70B shape.)
// Output: act[t][n] = mask[t][group of n] ? SiLU(gate) * up : 0, bf16, n = position in the union.
#include <type_traits>

#include "kernels.hpp"
#include "mask_words.hpp"
#include "row_stream.hpp"

namespace halo {

// T is a template parameter on purpose: with a run-time token count every (K piece, token) pair sat
// behind a branch of its own, each with its own wait for the LDS read in front of it, and the
// kernel spent more time on LDS latency than on memory (40 us at the 13B shape, 4 tokens).
template <int NCH, int T>
__global__ __launch_bounds__(256) void gate_up_ft(
    const bf16_t *__restrict__ x, int G, int gs, const bf16_t *__restrict__ Wg,
    const bf16_t *__restrict__ Wu, const uint8_t *__restrict__ mask, bf16_t *__restrict__ act, int act_stride,
    AheadPredDev ap)
{
    constexpr int TMAX = T;
    constexpr int d = NCH * 512, XR = d + 8;                 // LDS row of x, elements (16-byte aligned)
    extern __shared__ __attribute__((aligned(16))) bf16_t sx[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if ((int)blockIdx.x < ap.n_pred) {
        // paper Sec. III-B.3, Pred beside Load/Comp, one layer ahead: the next block's first layer
        predictor_row_tokens<d>(ap.x_next, ap.At, ap.h, T, d, ap.r, blockIdx.x * 4 + wave, lane);
        return;
    }
    // The token rows of x are requested first of all: they depend on nothing, so they travel beside the
    // mask bytes, and the weight rows requested after them never wait behind a staging round trip.
    constexpr int kPieces = T * (d / 8), kPer = (kPieces + 255) / 256;
    u32x4 xp[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int p = tid + 256 * j < kPieces ? tid + 256 * j : tid;
        const int t = p / (d / 8), e = (p - t * (d / 8)) * 8;
        xp[j] = *reinterpret_cast<const u32x4 *>(x + (size_t)t * d + e);
    }
    // the union of the tokens' surviving groups, built by every wave from the T*G mask bytes
    // (no separate launch, no list in memory between the mask and the first weight load)
    const MaskWords uw = load_union_words<TMAX>(mask, T, G, lane);
    const long long total = (long long)uw.count * gs;
    const int nw = (gridDim.x - ap.n_pred) * 4, w = (blockIdx.x - ap.n_pred) * 4 + wave;
    const int n0 = (int)(total * w / nw), n1 = (int)(total * (w + 1) / nw);
    const bool busy = n0 < n1;
    // a run is shorter than a group (total / nw <= gs), so it touches at most two groups: their ids
    // and the tokens' mask bits for them are fetched up front
    const int u_first = busy ? n0 / gs : 0, u_last = busy ? (n1 - 1) / gs : 0;
    const int g_first = uw.count ? nth_group(uw, u_first, lane) : 0, g_last = uw.count ? nth_group(uw, u_last, lane) : 0;
    auto row_of = [&](int n) -> size_t {
        const int u = n / gs;
        return (size_t)(u == u_first ? g_first : g_last) * gs + (n - u * gs);
    };
    unsigned keep_first = 0, keep_last = 0;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const unsigned a = mask[(size_t)t * G + g_first], b = mask[(size_t)t * G + g_last];
        keep_first |= (a ? 1u : 0u) << t;
        keep_last |= (b ? 1u : 0u) << t;
    }
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int p = tid + 256 * j;
        const int t = p / (d / 8), e = (p - t * (d / 8)) * 8;
        if (p < kPieces) *reinterpret_cast<u32x4 *>(sx + t * XR + e) = xp[j];
    }
    // the first two neurons' rows are on their way while the workgroup meets at the barrier
    RowPair<NCH> A, B;
    if (busy) load_rows<NCH>(A, Wg, Wu, row_of(n0), lane);
    if (n0 + 1 < n1) load_rows<NCH>(B, Wg, Wu, row_of(n0 + 1), lane);
    __syncthreads();
    if (!busy) return;                                       // no barrier below
    const bf16_t *xl = sx + lane * 8;
    // Reduces neuron n from the registers of r.  With `reload`, chunk k of row `next` is requested
    // into r as soon as the tokens have used chunk k of row n: the wave keeps close to two rows of
    // loads outstanding all the time, instead of one while it multiplies.
    auto finish = [&](RowPair<NCH> &r, int n, auto reload, size_t next) {
        float ag[TMAX], au[TMAX];
#pragma unroll
        for (int t = 0; t < TMAX; ++t) ag[t] = au[t] = 0.0f;
        const u32x4 *pg = reinterpret_cast<const u32x4 *>(Wg + next * d) + lane;
        const u32x4 *pu = reinterpret_cast<const u32x4 *>(Wu + next * d) + lane;
        // the tokens' pieces of chunk k + 1 are read from LDS while chunk k is multiplied
        u32x4 xv[2][T];
#pragma unroll
        for (int t = 0; t < T; ++t) xv[0][t] = *reinterpret_cast<const u32x4 *>(xl + t * XR);
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            if (k + 1 < NCH) {
#pragma unroll
                for (int t = 0; t < T; ++t)
                    xv[(k + 1) & 1][t] = *reinterpret_cast<const u32x4 *>(xl + t * XR + (k + 1) * 512);
                __builtin_amdgcn_sched_barrier(0);          // the reads go out before the multiply-adds
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const u32x4 &xk = xv[k & 1][t];
                ag[t] = dot2_bf16(r.g[k].x, xk.x, ag[t]);
                au[t] = dot2_bf16(r.u[k].x, xk.x, au[t]);
                ag[t] = dot2_bf16(r.g[k].y, xk.y, ag[t]);
                au[t] = dot2_bf16(r.u[k].y, xk.y, au[t]);
                ag[t] = dot2_bf16(r.g[k].z, xk.z, ag[t]);
                au[t] = dot2_bf16(r.u[k].z, xk.z, au[t]);
                ag[t] = dot2_bf16(r.g[k].w, xk.w, ag[t]);
                au[t] = dot2_bf16(r.u[k].w, xk.w, au[t]);
            }
            if constexpr (decltype(reload)::value) {
                r.g[k] = __builtin_nontemporal_load(pg + k * kWave);
                r.u[k] = __builtin_nontemporal_load(pu + k * kWave);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const unsigned keep = (n / gs == u_first) ? keep_first : keep_last;
        float mine = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const float v = silu_mul(wave_sum_fast(ag[t]), wave_sum_fast(au[t]));
            if (lane == t) mine = ((keep >> t) & 1u) ? v : 0.0f;
        }
        if (lane < T) act[(size_t)lane * act_stride + n] = f32_to_bf16(mine);
    };
    int n = n0;
    while (n + 3 < n1) {
        finish(A, n, std::true_type{}, row_of(n + 2));
        finish(B, n + 1, std::true_type{}, row_of(n + 3));
        n += 2;
    }
    // one, two or three neurons left; A holds n, B holds n + 1
    if (n + 2 < n1) {
        finish(A, n, std::true_type{}, row_of(n + 2));
        finish(B, n + 1, std::false_type{}, 0);
        finish(A, n + 2, std::false_type{}, 0);
    } else if (n + 1 < n1) {
        finish(A, n, std::false_type{}, 0);
        finish(B, n + 1, std::false_type{}, 0);
    } else {
        finish(A, n, std::false_type{}, 0);
    }
}

bool few_path_supported(int T, int d, int G, int gs)
{
    // up to 4 tokens: beyond that the 2*T multiply-adds per weight element no longer hide behind its
    // memory time (8 tokens at the 70B shape: 258 us against 150 us for the matrix-core kernel)
    return T >= 2 && T <= 4 && gs == 128 && G <= 256 && (d == 4096 || d == 5120 || d == 8192);
}

template <int NCH, int T>
static hipError_t launch_exact(const bf16_t *x, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                               const uint8_t *mask, bf16_t *act, int act_stride, hipStream_t s,
                               const AheadPredDev &ap)
{
    constexpr size_t lds = (size_t)T * (NCH * 512 + 8) * sizeof(bf16_t);
    static const hipError_t lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(gate_up_ft<NCH, T>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (lds_ok != hipSuccess) return lds_ok;
    launch_timed_lds("gate_up_ft", gate_up_ft<NCH, T>, dim3(256 + ap.n_pred), dim3(256), lds, s, x, G, gs, Wg, Wu,
                     mask, act, act_stride, ap);
    return hipGetLastError();
}

template <int NCH>
static hipError_t launch_one(const bf16_t *x, int T, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                             const uint8_t *mask, bf16_t *act, int act_stride, hipStream_t s,
                             const AheadPredDev &ap)
{
    switch (T) {
    case 2: return launch_exact<NCH, 2>(x, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    case 3: return launch_exact<NCH, 3>(x, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    case 4: return launch_exact<NCH, 4>(x, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gate_up_few(const bf16_t *x, int T, int d, int G, int gs, const bf16_t *Wg, const bf16_t *Wu,
                              const uint8_t *mask, bf16_t *act, int act_stride, hipStream_t s,
                              const AheadPredDev &ap)
{
    switch (d) {
    case 4096: return launch_one<8>(x, T, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    case 5120: return launch_one<10>(x, T, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    case 8192: return launch_one<16>(x, T, G, gs, Wg, Wu, mask, act, act_stride, s, ap);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace halo
