// Pieces shared by the two decode kernels (the vector-ALU one for fp32 / any group size and the
// bf16 matrix-core one): the map from logical cache entries to slots, and the partial record merge.
#pragma once

#include "common.h"

namespace sepattn {

// The state of one sequence's cache, read from its row of `sizes` and clamped so that no value can
// lead outside the buffers: counts of valid entries and the ring heads of the two ring regions.
//   slots [0,a) Initial Cache | [a,a+s) Separator Cache (ring) | [a+s,c) window (ring)
//   separator k (oldest first) sits in slot a + (sep_head + k) mod s,
//   window entry u (oldest first: Past Window, then Local Window) in slot a+s + (win_head + u) mod (c-a-s)
struct CacheMap {
    int n_init, n_sep, n_past, n_loc, sep_head, win_head, a, s, wcap;
};
__device__ inline CacheMap cache_map(const sepkv_params &p, const int32_t *__restrict__ sz) {
    CacheMap m;
    m.a = p.a;
    m.s = p.s;
    m.wcap = p.c - p.a - p.s;
    m.n_init = min(max(sz[0], 0), p.a);
    m.n_sep = min(max(sz[1], 0), p.s);
    m.n_past = min(max(sz[2], 0), m.wcap);
    m.n_loc = min(max(sz[3], 0), m.wcap - m.n_past);
    m.sep_head = p.s > 0 ? min(max(sz[4], 0), p.s - 1) : 0;
    m.win_head = min(max(sz[5], 0), m.wcap - 1);
    return m;
}
__device__ inline int sep_slot(const CacheMap &m, int k) {
    const int t = m.sep_head + k;
    return m.a + (t >= m.s ? t - m.s : t);
}
__device__ inline int win_index(const CacheMap &m, int u) {  // index into the window region (and its flag array)
    const int t = m.win_head + u;
    return t >= m.wcap ? t - m.wcap : t;
}
// logical valid entry e (oldest first over Initial, Separator, Past Window, Local Window) -> slot
__device__ inline int decode_slot_of(const CacheMap &m, int e) {
    if (e < m.n_init) return e;
    if (e < m.n_init + m.n_sep) return sep_slot(m, e - m.n_init);
    return m.a + m.s + win_index(m, e - m.n_init - m.n_sep);
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
