// Hand-over from prefill to the four-block KV cache (Sec. 3.2 "Generation" / Sec. 3.3): after a
// prompt of L tokens has been pre-filled, only the KV of the initial tokens, of the separators and of
// the neighbouring tokens is kept.  Per sequence the cache receives
//     Initial Cache    positions 0 .. min(a, L) - 1
//     Separator Cache  the newest (at most s) separators among the positions [min(a,L), L - nw),
//                      oldest first (older ones are dropped, as the compression step would)
//     window           the last nw positions; the newest min(w, nw) of them are the Local Window
// and sizes = (Size_init, Size_sep, nw - Size_local, Size_local, 0, 0) (both rings start at their first
// slot), win_is_sep = separator flag of each
// window entry.  Rows are copied bit-exactly.
//
// One kernel: a workgroup of 256 threads copies 16 (d = 128, bf16) rows per pass; blockIdx.y is the
// (sequence, KV head, K or V), blockIdx.x a run of kFillRows cache slots.  Workgroup x = 0 of KV
// head 0 / tensor K also writes the sequence's sizes and window flags.
#include "common.h"

namespace sepattn {

namespace {

constexpr int kFillThreads = 256;
constexpr int kFillRows = 128;  // cache slots per workgroup
constexpr int kFillUnroll = 8;  // rows a thread has in flight

__global__ __launch_bounds__(kFillThreads) void cache_fill_kernel(
    sepkv_params p, int L, int nw, int cap, int row16, const uint4 *__restrict__ K, const uint4 *__restrict__ V,
    const uint8_t *__restrict__ is_sep, const int32_t *__restrict__ sep_idx, const int32_t *__restrict__ sep_prefix,
    uint4 *__restrict__ Kc, uint4 *__restrict__ Vc, uint8_t *__restrict__ win_is_sep, int32_t *__restrict__ sizes) {
    const int which = blockIdx.y & 1;
    const int kv = (blockIdx.y >> 1) % p.Hkv;
    const int sq = (blockIdx.y >> 1) / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)sq * (L + 1);
    const int32_t *idx = sep_idx + (long)sq * cap;
    const int n_init = min(p.a, L);
    const int wstart = L - nw;                       // first window position; >= n_init (host check)
    const int seps_before = prefix[wstart];          // separators at positions < wstart
    const int n_old = seps_before - prefix[n_init];  // ... that are not initial tokens
    const int kept = min(min(p.s, n_old), max(cap - (seps_before - min(p.s, n_old)), 0));  // listed ones only
    const int first_kept = seps_before - min(p.s, n_old);
    const int wcap = p.c - p.a - p.s;

    if (blockIdx.x == 0 && kv == 0 && which == 0) {
        const int wl = min(p.w, nw);
        if (threadIdx.x == 0) {
            int32_t *sz = sizes + SEPKV_SIZES_COLS * sq;
            sz[0] = n_init;
            sz[1] = kept;
            sz[2] = nw - wl;
            sz[3] = wl;
            sz[4] = 0;  // both rings start at their first slot
            sz[5] = 0;
        }
        for (int u = threadIdx.x; u < nw; u += kFillThreads) win_is_sep[(long)sq * wcap + u] = is_sep[(long)sq * L + wstart + u];
    }

    const uint4 *src = (which ? V : K) + ((long)sq * p.Hkv + kv) * (long)L * row16;
    uint4 *dst = (which ? Vc : Kc) + ((long)sq * p.Hkv + kv) * (long)p.c * row16;
    const int rows_per_pass = kFillThreads / row16;
    const int r_in = threadIdx.x / row16, piece = threadIdx.x % row16;
    const int t_end = min((int)(blockIdx.x + 1) * kFillRows, p.c);
    // A pure gather-copy: what limits it is how many loads a thread keeps in flight.  A thread handles
    // kFillUnroll rows at a time: first all their source positions (for separator slots a dependent
    // load from the compacted list), then all row loads, then all stores.
    for (int t0 = blockIdx.x * kFillRows; t0 < t_end; t0 += rows_per_pass * kFillUnroll) {
        int jsrc[kFillUnroll];  // source position of the slot, -1: the slot stays as it is
#pragma unroll
        for (int u = 0; u < kFillUnroll; ++u) {
            const int t = t0 + u * rows_per_pass + r_in;  // cache slot
            int j = -1;
            if (t < t_end) {
                if (t < p.a) {
                    if (t < n_init) j = t;
                } else if (t < p.a + p.s) {
                    const int k = t - p.a;
                    // the clamp keeps a stale list entry (caller broke sep_count <= cap) from faulting
                    if (k < kept) j = min(max(idx[first_kept + k], 0), L - 1);
                } else {
                    const int u_w = t - p.a - p.s;
                    if (u_w < nw) j = wstart + u_w;
                }
            }
            jsrc[u] = j;
        }
        uint4 v[kFillUnroll];
        // every row is read once and written once: non-temporal on both sides
#pragma unroll
        for (int u = 0; u < kFillUnroll; ++u)
            if (jsrc[u] >= 0) v[u] = nt_load(&src[(long)jsrc[u] * row16 + piece]);
#pragma unroll
        for (int u = 0; u < kFillUnroll; ++u) {
            const int t = t0 + u * rows_per_pass + r_in;
            if (jsrc[u] >= 0) nt_store(v[u], &dst[(long)t * row16 + piece]);
        }
    }
}

}  // namespace

int launch_cache_fill(const sepkv_params &p, int L, int nw, const void *K, const void *V, const uint8_t *is_sep,
                      const int32_t *sep_idx, int cap, const int32_t *sep_prefix, void *Kc, void *Vc,
                      uint8_t *win_is_sep, int32_t *sizes, hipStream_t st) {
    const int elem = (p.dtype == SEPATTN_BF16) ? 2 : 4;
    const int row16 = p.d * elem / 16;
    const long ny = (long)p.S * p.Hkv * 2;
    if (ny > 65535L) return SEPATTN_ERR_SHAPE;
    dim3 grid((p.c + kFillRows - 1) / kFillRows, (unsigned)ny);
    ProfScope prof(SEPATTN_K_CACHE_FILL, st);
    hipLaunchKernelGGL(cache_fill_kernel, grid, dim3(kFillThreads), 0, st, p, L, nw, cap, row16,
                       static_cast<const uint4 *>(K), static_cast<const uint4 *>(V), is_sep, sep_idx, sep_prefix,
                       static_cast<uint4 *>(Kc), static_cast<uint4 *>(Vc), win_is_sep, sizes);
    return launch_status();
}

}  // namespace sepattn
