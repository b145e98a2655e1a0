// Semantic-aware predictor (paper Sec. III-B.2): h = ReLU(x A), scores = h B.
//
// Both layers are the same operation, out[t][j] = f(dot(X[t], W[j])), with the
// float32 summation order fixed so that the ranking derived from the scores is
// reproducible bit for bit: element i goes to partial sum (i/8) mod 64 (one
// partial per lane of a wave64, eight consecutive elements = one 16-byte bf16
// load), each partial is a fused-multiply-add chain in increasing i starting at
// +0, and the 64 partials are combined by a butterfly at distances 32..1.
// The work is plain float ALU on purpose: a matrix-core instruction would not
// expose its internal summation order.
#include "kernels.hpp"

namespace halo {

template <typename XT, typename WT, bool RELU>
__global__ __launch_bounds__(256) void dot_rows_kernel(const XT *__restrict__ X,
                                                       const WT *__restrict__ W,
                                                       float *__restrict__ out, int T, int R, int n)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long idx = (long long)blockIdx.x * 4 + wave;
    if (idx >= (long long)T * R) return;                 // uniform per wave
    const int t = (int)(idx / R), j = (int)(idx % R);
    const float p = dot_order64(X + (size_t)t * n, W + (size_t)j * n, n, lane);
    if (lane == 0) out[idx] = RELU ? (p > 0.0f ? p : 0.0f) : p;
}

// First layer for many tokens, bf16, d = NCH*512: a wave keeps JB rows of At in registers
// (as floats) and sweeps a range of tokens, so At is read once per 32 tokens instead of once
// per token.  Same arithmetic per (token, row) as dot_order64: lane l owns the 8-element
// pieces l, l+64, ... in increasing order, one fused-multiply-add chain from +0, butterfly.
constexpr int kPredTokens = 32;     // tokens per workgroup (64: 44 us, 32: 29 us, 16: 32 us at 512 tokens, 7B shape)

template <int NCH, int JB, int TB>
__global__ __launch_bounds__(256) void hidden_rows_kernel(const bf16_t *__restrict__ X,
                                                          const bf16_t *__restrict__ At,
                                                          float *__restrict__ h, int T, int r)
{
    constexpr int d = NCH * 512;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j0 = (blockIdx.x * 4 + wave) * JB;
    if (j0 >= r) return;
    float wr[JB][NCH][8];
#pragma unroll
    for (int b = 0; b < JB; ++b) {
        const int j = j0 + b < r ? j0 + b : r - 1;
#pragma unroll
        for (int k = 0; k < NCH; ++k) load8(At + (size_t)j * d + (k * kWave + lane) * 8, wr[b][k]);
    }
    const int t0 = blockIdx.y * kPredTokens, t1 = min(T, t0 + kPredTokens);
    // TB tokens per iteration; the next iteration's x pieces are requested before the current
    // ones are used, so the sweep is not one memory round trip per token
    auto fetch = [&](u32x4 (&xv)[TB][NCH], int t) {
#pragma unroll
        for (int c = 0; c < TB; ++c) {
            const int tc = t + c < t1 ? t + c : t1 - 1;          // past the end: a duplicate, not stored
#pragma unroll
            for (int k = 0; k < NCH; ++k)
                xv[c][k] = *reinterpret_cast<const u32x4 *>(X + (size_t)tc * d + (k * kWave + lane) * 8);
        }
    };
    auto finish = [&](const u32x4 (&xv)[TB][NCH], int t) {
        float p[TB][JB];
#pragma unroll
        for (int c = 0; c < TB; ++c)
#pragma unroll
            for (int b = 0; b < JB; ++b) p[c][b] = 0.0f;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
#pragma unroll
            for (int c = 0; c < TB; ++c) {
                float xf[8];
                unpack8(xv[c][k], xf);
#pragma unroll
                for (int b = 0; b < JB; ++b)
#pragma unroll
                    for (int e = 0; e < 8; ++e) p[c][b] = __builtin_fmaf(xf[e], wr[b][k][e], p[c][b]);
            }
        }
#define HALO_STEP(OFF)                                               \
    _Pragma("unroll") for (int c = 0; c < TB; ++c)                   \
        _Pragma("unroll") for (int b = 0; b < JB; ++b) p[c][b] = xor_add<OFF>(p[c][b]);
        HALO_STEP(32) HALO_STEP(16) HALO_STEP(8) HALO_STEP(4) HALO_STEP(2) HALO_STEP(1)
#undef HALO_STEP
        if (lane == 0) {
#pragma unroll
            for (int c = 0; c < TB; ++c)
#pragma unroll
                for (int b = 0; b < JB; ++b)
                    if (t + c < t1 && j0 + b < r)
                        h[(size_t)(t + c) * r + j0 + b] = p[c][b] > 0.0f ? p[c][b] : 0.0f;
        }
    };
    u32x4 xa[TB][NCH], xb[TB][NCH];
    fetch(xa, t0);
    int t = t0;
    for (; t + 2 * TB < t1; t += 2 * TB) {      // two iterations per trip: the buffers swap by name
        fetch(xb, t + TB);
        finish(xa, t);
        fetch(xa, t + 2 * TB);
        finish(xb, t + TB);
    }
    if (t + TB < t1) {
        fetch(xb, t + TB);
        finish(xa, t);
        finish(xb, t + TB);
    } else {
        finish(xa, t);
    }
}

template <int NCH, int JB, int TB>
static void launch_hidden_rows(const bf16_t *x, int T, int r, const bf16_t *At, float *h, hipStream_t s)
{
    hidden_rows_kernel<NCH, JB, TB><<<dim3((r + 4 * JB - 1) / (4 * JB), (T + kPredTokens - 1) / kPredTokens),
                                     dim3(256), 0, s>>>(x, At, h, T, r);
}

static bool hidden_rows_tiled(const bf16_t *x, int T, int d, int r, const bf16_t *At, float *h, hipStream_t s)
{
    if (T < 16) return false;
    switch (d) {
    case 4096: launch_hidden_rows<8, 2, 1>(x, T, r, At, h, s); return true;
    case 5120: launch_hidden_rows<10, 2, 1>(x, T, r, At, h, s); return true;
    case 8192: launch_hidden_rows<16, 1, 1>(x, T, r, At, h, s); return true;
    default: return false;
    }
}
static bool hidden_rows_tiled(const float *, int, int, int, const float *, float *, hipStream_t) { return false; }

template <typename WT>
static hipError_t predict_t(const WT *x, int T, int d, int r, int G, const WT *At, const WT *Bt,
                            float *h, float *scores, hipStream_t s)
{
    long long n1 = (long long)T * r, n2 = (long long)T * G;
    if (!hidden_rows_tiled(x, T, d, r, At, h, s))
        dot_rows_kernel<WT, WT, true><<<dim3((unsigned)((n1 + 3) / 4)), dim3(256), 0, s>>>(x, At, h, T, r, d);
    if (scores)
        dot_rows_kernel<float, WT, false><<<dim3((unsigned)((n2 + 3) / 4)), dim3(256), 0, s>>>(h, Bt, scores, T, G, r);
    return hipGetLastError();
}

// scores == nullptr: first layer only (h), the second layer is then fused into the mask kernel
hipError_t launch_predictor(int dtype, const void *x, int T, int d, int r, int G, const void *At,
                            const void *Bt, float *h, float *scores, hipStream_t s)
{
    if (dtype == 0)
        return predict_t<float>((const float *)x, T, d, r, G, (const float *)At, (const float *)Bt, h, scores, s);
    return predict_t<bf16_t>((const bf16_t *)x, T, d, r, G, (const bf16_t *)At, (const bf16_t *)Bt, h, scores, s);
}

}  // namespace halo
