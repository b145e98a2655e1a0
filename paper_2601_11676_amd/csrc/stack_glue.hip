// Harness aid (not part of the paper's method): the glue between the blocks of an FFN-only stack,
//     h[t] += y[t];   x[t] = h[t] / sqrt(mean(h[t]^2) + eps)
// in one launch, so that a benchmark of a whole stack spends one small kernel per layer on it
// instead of a chain of elementwise library kernels.  h is the float32 residual stream; y and x
// have the stack's element type.  One workgroup per token.
#include "../../include/halo.h"

#include "kernels.hpp"

namespace halo {
namespace {

template <typename WT>
__global__ __launch_bounds__(256) void residual_norm_kernel(float *__restrict__ h, const WT *__restrict__ y,
                                                            WT *__restrict__ x, int d, float eps)
{
    __shared__ float s_part[4];
    const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float *ht = h + (size_t)t * d;
    float sq = 0.0f;
    for (int i = tid; i < d; i += 256) {
        float v = ht[i];
        if (y) {
            v += to_float(y[(size_t)t * d + i]);
            ht[i] = v;
        }
        sq = __builtin_fmaf(v, v, sq);
    }
    sq = wave_sum(sq);
    if (lane == 0) s_part[wave] = sq;
    __syncthreads();
    const float total = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
    const float scale = 1.0f / sqrtf(total / (float)d + eps);
    for (int i = tid; i < d; i += 256) store_out(x + (size_t)t * d + i, ht[i] * scale);
}

}  // namespace
}  // namespace halo

extern "C" int halo_stack_residual_norm(float *h, const void *y, void *x, int32_t T, int32_t d, int32_t dtype,
                                        float eps, void *stream)
{
    using namespace halo;
    if (!h || !x) return HALO_ERR_NULL;
    if (dtype != HALO_F32 && dtype != HALO_BF16) return HALO_ERR_DTYPE;
    if (T < 0 || d < 1 || !(eps >= 0.0f)) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == HALO_F32)
        residual_norm_kernel<float><<<dim3(T), dim3(256), 0, s>>>(h, (const float *)y, (float *)x, d, eps);
    else
        residual_norm_kernel<bf16_t><<<dim3(T), dim3(256), 0, s>>>(h, (const bf16_t *)y, (bf16_t *)x, d, eps);
    return hipGetLastError() == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}
