// Group mask (paper Sec. III-B.3): importance rank -> priority index -> device -> survivors.
//
// One workgroup per token.  The ranking is by counting: the rank of group g is the
// number of groups that come before it under (score descending, lower index first on
// equal scores, NaN after every number).  G <= 1024, so G^2 compares per token is
// small, needs no sort network and gives each group its rank independently.
#include "kernels.hpp"

namespace halo {

__device__ __forceinline__ bool ranks_before(float sh, int h, float sg, int g)
{
    const bool nh = sh != sh, ng = sg != sg;
    if (nh | ng) return (nh & ng) ? (h < g) : ng;
    return (sh > sg) | ((sh == sg) & (h < g));
}

__global__ __launch_bounds__(256) void group_mask_kernel(
    const float *__restrict__ scores, int G, int K, const int8_t *__restrict__ prio_dev, int n_dev,
    const uint8_t *__restrict__ drop, int32_t *__restrict__ order, int8_t *__restrict__ group_dev,
    uint8_t *__restrict__ mask, int32_t *__restrict__ surv_idx, int32_t *__restrict__ n_surv)
{
    __shared__ float s_score[1024];
    __shared__ uint8_t s_mask[1024];
    const int t = blockIdx.x, tid = threadIdx.x;
    for (int g = tid; g < G; g += 256) s_score[g] = scores[(size_t)t * G + g];
    __syncthreads();
    for (int g = tid; g < G; g += 256) {
        const float sg = s_score[g];
        int pos = 0;
        for (int h = 0; h < G; ++h) pos += ranks_before(s_score[h], h, sg, g) ? 1 : 0;
        if (order) order[(size_t)t * G + pos] = g;
        int dev = -1;
        uint8_t m = 0;
        if (pos < K) {
            dev = prio_dev[pos];
            if (dev >= 0 && dev < n_dev) {
                m = (drop && drop[(size_t)t * n_dev + dev]) ? 0 : 1;
            } else {
                dev = -1;   // malformed schedule entry: treated as not executed
            }
        }
        if (group_dev) group_dev[(size_t)t * G + g] = (int8_t)dev;
        mask[(size_t)t * G + g] = m;
        s_mask[g] = m;
    }
    __syncthreads();
    int total = 0;
    for (int h = 0; h < G; ++h) total += s_mask[h];
    if (tid == 0 && n_surv) n_surv[t] = total;
    if (surv_idx) {
        for (int g = tid; g < G; g += 256) {
            if (!s_mask[g]) continue;
            int c = 0;
            for (int h = 0; h < g; ++h) c += s_mask[h];
            surv_idx[(size_t)t * K + c] = g;
        }
        for (int p = total + tid; p < K; p += 256) surv_idx[(size_t)t * K + p] = -1;
    }
}

hipError_t launch_group_mask(const float *scores, int T, int G, int K, const int8_t *prio_dev,
                             int n_dev, const uint8_t *drop, int32_t *order, int8_t *group_dev,
                             uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s)
{
    group_mask_kernel<<<dim3(T), dim3(256), 0, s>>>(scores, G, K, prio_dev, n_dev, drop, order,
                                                    group_dev, mask, surv_idx, n_surv);
    return hipGetLastError();
}

}  // namespace halo
