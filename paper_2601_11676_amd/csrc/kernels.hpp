// Internal launcher interface between the C boundary (halo_api.hip) and the kernels.
#pragma once
#include "common.hpp"

namespace halo {

// predictor.hip
hipError_t launch_predictor(int dtype, const void *x, int T, int d, int r, int G, const void *At,
                            const void *Bt, float *h, float *scores, hipStream_t s);

// mask.hip
hipError_t launch_group_mask(const float *scores, int T, int G, int K, const int8_t *prio_dev,
                             int n_dev, const uint8_t *drop, int32_t *order, int8_t *group_dev,
                             uint8_t *mask, int32_t *surv_idx, int32_t *n_surv, hipStream_t s);

// ffn_decode.hip : float-ALU paths (any T; tuned for one token)
struct DecodeScratch {
    int32_t *ulist;     // [G]   groups surviving for at least one token, ascending
    int32_t *meta;      // [16 + ...] meta[0] = |ulist|; meta[16..] arrival counters
    float *act;         // [T][ffn] activations SiLU(gate)*up, compacted by union slot
    float *partial;     // [n_split][T][d] partial down-projection sums
    int n_split;        // neuron subsets in the down projection
};
int decode_n_split(int T, int d);
hipError_t launch_ffn_decode(int dtype, const void *x, int T, int d, int G, int gs, const void *Wg,
                             const void *Wu, const void *WdT, const uint8_t *mask, void *y,
                             const DecodeScratch &ws, hipStream_t s);

}  // namespace halo
