// Internal declarations shared by the HIP sources of libsepattn (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sepattn.h"

namespace sepattn {

constexpr int kWave = 64;

inline int launch_status() { return hipGetLastError() == hipSuccess ? SEPATTN_OK : SEPATTN_ERR_HIP; }
// An error that an earlier, unrelated runtime call of the caller left pending would otherwise be read
// (and blamed on this call) by the first launch_status(): every entry point discards it first.
inline void discard_stale_hip_error() { (void)hipGetLastError(); }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// 16-byte loads and stores with the non-temporal hint, for rows that are touched once
typedef unsigned int nt_u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 nt_load(const uint4 *p) {
    const nt_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline void nt_store(uint4 v, uint4 *p) {
    const nt_u32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<nt_u32x4 *>(p));
}

// number of compute units of the current device (queried once per device; 256 if the query fails)
int compute_units();

// Measurement hook: brackets launches of the selected kernel with HIP events (see sepattn.h).
void profile_mark(int kernel, hipStream_t st, bool stop);
struct ProfScope {
    int kernel;
    hipStream_t st;
    ProfScope(int k, hipStream_t s) : kernel(k), st(s) { profile_mark(kernel, st, false); }
    ~ProfScope() { profile_mark(kernel, st, true); }
};

// Head-wise neighbour windows (the head-wise variant of Sec. 4.6): every attention kernel runs with
// p.n = the LARGEST window of the call and gets, by value, how much shorter each query head's own
// window is.  The key streams and the far / band split are those of the largest window (so heads
// that share K/V tiles still share them); only the visibility test of a band key uses the head's
// own window:  key j, not an initial token or a separator, is visible to query i of head h iff
// j <= i <= j + p.n - 1 - delta[h].  All zeros for an ordinary call.
constexpr int kMaxHeadwise = SEPATTN_MAX_HEADWISE_HEADS;
struct HeadWin {
    int32_t delta[kMaxHeadwise];
};
__host__ __device__ inline int head_delta(const HeadWin &hw, int h) {
    return hw.delta[h < kMaxHeadwise ? h : kMaxHeadwise - 1];
}

// ---- integer kernels -------------------------------------------------------------------------
struct SepIdSet {
    int n;
    int ids[SEPATTN_MAX_SEP_IDS];
};
int launch_mark(const int32_t *token_ids, long n_tokens, const SepIdSet &set, uint8_t *is_sep,
                hipStream_t st);
int launch_mark_interval(int B, int L, int delta, int phase, uint8_t *is_sep, hipStream_t st);
constexpr int kCompactChunk = 2048;  // tokens per workgroup of the compaction kernels
int launch_compact(const uint8_t *is_sep, int B, int L, int32_t *sep_idx, int cap,
                   int32_t *sep_count, int32_t *sep_prefix, int32_t *chunk_counts, hipStream_t st);
int launch_mark_compact(const int32_t *token_ids, int B, int L, const SepIdSet &set, uint8_t *is_sep,
                        int32_t *sep_idx, int cap, int32_t *sep_count, int32_t *sep_prefix,
                        int32_t *chunk_counts, hipStream_t st);

// ---- fp32 debug path ---------------------------------------------------------------------------
// doc_start / doc_end: packed documents (per-position bounds [B, L]), or nullptr
int launch_forward_fp32(const sepattn_params &p, const HeadWin &hw, const float *Q, const float *K, const float *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, const int32_t *doc_start, float *O,
                        float *LSE, hipStream_t st);
int launch_backward_fp32(const sepattn_params &p, const HeadWin &hw, const float *Q, const float *K, const float *V,
                         const float *O, const float *LSE, const float *dO, const int32_t *sep_idx,
                         const int32_t *sep_prefix, const int32_t *doc_start, const int32_t *doc_end, float *dQ,
                         float *dK, float *dV, float *Dws, hipStream_t st);

// ---- bf16 MFMA path ----------------------------------------------------------------------------
size_t forward_bf16_workspace(const sepattn_params &p);
// doc_start / doc_end: packed documents (per-position bounds [B, L]; p.a must be 0), or nullptr
int launch_forward_bf16(const sepattn_params &p, const HeadWin &hw, const void *Q, const void *K, const void *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, const int32_t *doc_start,
                        const int32_t *doc_end, void *O, float *LSE, void *ws, hipStream_t st);
int launch_doc_bounds(const int32_t *cu_seqlens, int n_docs, int L, int a, int32_t *doc_start, int32_t *doc_end,
                      uint8_t *is_sep, hipStream_t st);
size_t backward_bf16_workspace(const sepattn_params &p);
int launch_backward_bf16(const sepattn_params &p, const HeadWin &hw, const void *Q, const void *K, const void *V,
                         const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                         const int32_t *sep_count, const int32_t *sep_prefix, const int32_t *doc_start,
                         const int32_t *doc_end, void *dQ, void *dK, void *dV, void *ws, hipStream_t st);

// ---- streaming cache ---------------------------------------------------------------------------
int check_kv_params(const sepkv_params *p);  // host validation shared by every cache call
size_t decode_workspace(const sepkv_params &p);
// rope: table of cos / sin by position [n_pos][2][d/2] (keys stored without position encoding), or nullptr
int launch_decode(const sepkv_params &p, const void *q, const void *Kc, const void *Vc,
                  const int32_t *sizes, const float *rope, int n_pos, void *out, float *lse, void *ws,
                  hipStream_t st);
int launch_rope_table(int n_pos, int d, double base, float *table, hipStream_t st);
int launch_cache_append(const sepkv_params &p, const void *k_new, const void *v_new, const uint8_t *is_sep_new,
                        void *Kc, void *Vc, uint8_t *win_is_sep, int32_t *sizes, hipStream_t st);
size_t evict_workspace(const sepkv_params &p);
int launch_evict(const sepkv_params &p, void *Kc, void *Vc, const uint8_t *win_is_sep, int32_t *sizes,
                 void *ws, hipStream_t st);
int launch_cache_fill(const sepkv_params &p, int L, int nw, const void *K, const void *V, const uint8_t *is_sep,
                      const int32_t *sep_idx, int cap, const int32_t *sep_prefix, void *Kc, void *Vc,
                      uint8_t *win_is_sep, int32_t *sizes, hipStream_t st);

}  // namespace sepattn
