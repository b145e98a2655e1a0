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

template <typename WT>
static hipError_t predict_t(const WT *x, int T, int d, int r, int G, const WT *At, const WT *Bt,
                            float *h, float *scores, hipStream_t s)
{
    long long n1 = (long long)T * r, n2 = (long long)T * G;
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
