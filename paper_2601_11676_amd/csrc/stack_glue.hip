// Harness aid (not part of the paper's method): the glue between the blocks of an FFN-only stack,
//     h[t] += y[t];   x[t] = h[t] / sqrt(mean(h[t]^2) + eps)
// in one launch, so that a benchmark of a whole stack spends one small kernel per layer on it
// instead of a chain of elementwise library kernels.  h is the float32 residual stream; y and x
// have the stack's element type.  One workgroup per token.
#include "../../include/halo.h"

#include "kernels.hpp"

namespace halo {
namespace {

// A thread keeps its elements in registers between the sum of squares and the scaling: chunk c of a
// thread is the four elements (c * 256 + tid) * 4 .. + 3, all loads of a row go out together.
constexpr int kGlueChunks = 8;                       // 256 threads x 8 chunks x 4 elements = rows up to 8192

__device__ __forceinline__ float4 load4f(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 load4f(const bf16_t *p)
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    return make_float4(bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y));
}
__device__ __forceinline__ void store4(float *p, const float4 &v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ void store4(bf16_t *p, const float4 &v)
{
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
    o.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
    *reinterpret_cast<uint2 *>(p) = o;
}

template <typename WT>
__global__ __launch_bounds__(256) void residual_norm_kernel(float *__restrict__ h, const WT *__restrict__ y,
                                                            WT *__restrict__ x, int d, float eps)
{
    __shared__ float s_part[4];
    const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float *ht = h + (size_t)t * d;
    float4 v[kGlueChunks], w[kGlueChunks];
#pragma unroll
    for (int c = 0; c < kGlueChunks; ++c) {
        const int e = (c * 256 + tid) * 4;
        v[c] = e < d ? load4f(ht + e) : make_float4(0.f, 0.f, 0.f, 0.f);
        w[c] = (y && e < d) ? load4f(y + (size_t)t * d + e) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float sq = 0.0f;
#pragma unroll
    for (int c = 0; c < kGlueChunks; ++c) {
        v[c].x += w[c].x;
        v[c].y += w[c].y;
        v[c].z += w[c].z;
        v[c].w += w[c].w;
        sq = __builtin_fmaf(v[c].x, v[c].x, sq);
        sq = __builtin_fmaf(v[c].y, v[c].y, sq);
        sq = __builtin_fmaf(v[c].z, v[c].z, sq);
        sq = __builtin_fmaf(v[c].w, v[c].w, sq);
        const int e = (c * 256 + tid) * 4;
        if (y && e < d) store4(ht + e, v[c]);
    }
    sq = wave_sum(sq);
    if (lane == 0) s_part[wave] = sq;
    __syncthreads();
    const float total = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
    const float scale = 1.0f / sqrtf(total / (float)d + eps);
#pragma unroll
    for (int c = 0; c < kGlueChunks; ++c) {
        const int e = (c * 256 + tid) * 4;
        if (e < d) store4(x + (size_t)t * d + e, make_float4(v[c].x * scale, v[c].y * scale, v[c].z * scale, v[c].w * scale));
    }
}

}  // namespace
}  // namespace halo

extern "C" int halo_stack_residual_norm(float *h, const void *y, void *x, int32_t T, int32_t d, int32_t dtype,
                                        float eps, void *stream)
{
    using namespace halo;
    if (!h || !x) return HALO_ERR_NULL;
    if (dtype != HALO_F32 && dtype != HALO_BF16) return HALO_ERR_DTYPE;
    if (T < 0 || d < 4 || d % 4 || d > 256 * 4 * kGlueChunks || !(eps >= 0.0f)) return HALO_ERR_ARG;
    if (T == 0) return HALO_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == HALO_F32)
        residual_norm_kernel<float><<<dim3(T), dim3(256), 0, s>>>(h, (const float *)y, (float *)x, d, eps);
    else
        residual_norm_kernel<bf16_t><<<dim3(T), dim3(256), 0, s>>>(h, (const bf16_t *)y, (bf16_t *)x, d, eps);
    return hipGetLastError() == hipSuccess ? HALO_OK : HALO_ERR_HIP;
}
