// Group mask (paper Sec. III-B.3): importance rank -> priority index -> device -> survivors.
// One workgroup per token; the work itself is in mask_device.hpp.
//
// mask_scores_kernel optionally computes the scores itself (second predictor layer,
// paper Sec. III-B.2, same fixed-order dot product as predictor.hip) so that the fused
// pass saves a launch; the arithmetic is shared, so the bits are the same.
#include "kernels.hpp"
#include "mask_device.hpp"

namespace halo {

constexpr int kMaskThreads = 1024;

template <typename WT, bool FUSED_SCORES, int NT = kMaskThreads>
__global__ __launch_bounds__(NT) void mask_scores_kernel(
    const float *__restrict__ h, const WT *__restrict__ Bt, int r,      // FUSED_SCORES only
    float *__restrict__ scores, int G, int K, const int8_t *__restrict__ prio_dev, int n_dev,
    const uint8_t *__restrict__ drop, int32_t *__restrict__ order, int8_t *__restrict__ group_dev,
    uint8_t *__restrict__ mask, int32_t *__restrict__ surv_idx, int32_t *__restrict__ n_surv)
{
    __shared__ MaskShared sh;
    const size_t t = blockIdx.x;
    mask_scores_block<NT, WT, FUSED_SCORES>(
        sh, threadIdx.x, FUSED_SCORES ? h + t * r : nullptr, Bt, r, scores + t * G, G, K, prio_dev, n_dev,
        drop ? drop + t * n_dev : nullptr, order ? order + t * G : nullptr,
        group_dev ? group_dev + t * G : nullptr, mask + t * G, surv_idx ? surv_idx + t * K : nullptr,
        n_surv ? n_surv + t : nullptr);
}

hipError_t launch_group_mask(const float *scores, int T, int G, int K, const int8_t *prio_dev,
                             int n_dev, const uint8_t *drop, int32_t *order, int8_t *group_dev,
                             uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s)
{
    mask_scores_kernel<float, false><<<dim3(T), dim3(kMaskThreads), 0, s>>>(
        nullptr, nullptr, 0, const_cast<float *>(scores), G, K, prio_dev, n_dev, drop, order,
        group_dev, mask, surv_idx, n_surv);
    return hipGetLastError();
}

hipError_t launch_scores_and_mask(int dtype, const float *h, const void *Bt, int r, float *scores,
                                  int T, int G, int K, const int8_t *prio_dev, int n_dev,
                                  const uint8_t *drop, int32_t *order, int8_t *group_dev,
                                  uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s)
{
    if (dtype == 0)
        mask_scores_kernel<float, true><<<dim3(T), dim3(kMaskThreads), 0, s>>>(
            h, (const float *)Bt, r, scores, G, K, prio_dev, n_dev, drop, order, group_dev, mask,
            surv_idx, n_surv);
    else if (T >= 64)
        // many tokens: workgroups of 512 threads, more of them resident per compute unit (measured at
        // 512 tokens of the 7B shape: 11.5 us against 13.6 us with 1024 threads and 14.7 us with 256)
        mask_scores_kernel<bf16_t, true, 512><<<dim3(T), dim3(512), 0, s>>>(
            h, (const bf16_t *)Bt, r, scores, G, K, prio_dev, n_dev, drop, order, group_dev, mask,
            surv_idx, n_surv);
    else
        mask_scores_kernel<bf16_t, true><<<dim3(T), dim3(kMaskThreads), 0, s>>>(
            h, (const bf16_t *)Bt, r, scores, G, K, prio_dev, n_dev, drop, order, group_dev, mask,
            surv_idx, n_surv);
    return hipGetLastError();
}

}  // namespace halo
