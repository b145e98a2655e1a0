// A neuron's gate row and up row (bf16, d = NCH*512) held in registers as they were loaded:
// shared by the kernels that stream weight rows one wave per neuron.
#pragma once
#include "common.hpp"

namespace halo {

template <int NCH>
struct RowPair {
    u32x4 g[NCH], u[NCH];
};

template <int NCH>
__device__ __forceinline__ void load_rows(RowPair<NCH> &r, const bf16_t *__restrict__ Wg,
                                          const bf16_t *__restrict__ Wu, size_t row, int lane)
{
    constexpr int d = NCH * 512;
    const u32x4 *pg = reinterpret_cast<const u32x4 *>(Wg + row * d) + lane;
    const u32x4 *pu = reinterpret_cast<const u32x4 *>(Wu + row * d) + lane;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        r.g[k] = __builtin_nontemporal_load(pg + k * kWave);
        r.u[k] = __builtin_nontemporal_load(pu + k * kWave);
    }
}

}  // namespace halo
