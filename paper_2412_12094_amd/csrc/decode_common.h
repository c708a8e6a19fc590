// Pieces shared by the two decode kernels (the vector-ALU one for fp32 / any group size and the
// bf16 matrix-core one): the map from logical cache entries to slots, and the partial record merge.
#pragma once

#include "common.h"

namespace sepattn {

// logical valid entry e -> physical cache slot: [0,a) initial | [a,a+s) separator | [a+s,c) window
__device__ inline int decode_slot_of(int e, int n_init, int n_sep, int a, int s) {
    if (e < n_init) return e;
    if (e < n_init + n_sep) return a + (e - n_init);
    return a + s + (e - n_init - n_sep);
}

__device__ inline uint16_t decode_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

bool decode_mfma_applicable(const sepkv_params &p);
int decode_mfma_nsplit(const sepkv_params &p);
// rope: table of cos / sin by position [n_pos][2][d/2], or nullptr for keys that carry their encoding
int launch_decode_mfma(const sepkv_params &p, int nsplit, const uint16_t *q, const uint16_t *Kc, const uint16_t *Vc,
                       const int32_t *sizes, const float *rope, int n_pos, uint16_t *out, float *lse, float *part,
                       hipStream_t st);

}  // namespace sepattn
