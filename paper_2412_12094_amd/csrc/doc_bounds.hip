// Packed documents: per-position document bounds from the cumulative lengths, and the documents'
// initial tokens added to the marker bitmap.  Every document of a packed row is a sequence of its
// own (Sec. 3.1: its first a tokens are its initial tokens); with those tokens marked like
// separators the attention kernels need only the two bounds per position and run with a = 0.
#include "common.h"

namespace sepattn {

namespace {

__global__ __launch_bounds__(256) void doc_bounds_kernel(const int32_t *__restrict__ cu, int n_docs, int L, int a,
                                                         int32_t *__restrict__ doc_start,
                                                         int32_t *__restrict__ doc_end,
                                                         uint8_t *__restrict__ is_sep) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= L) return;
    // largest k in [0, n_docs) with cu[k] <= i (cu[0] = 0 by contract; a broken array cannot fault:
    // k stays in range and the bounds are clamped around i)
    int lo = 0, hi = n_docs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (cu[mid] <= i)
            lo = mid;
        else
            hi = mid - 1;
    }
    const int s = min(max(cu[lo], 0), i), e = min(max(cu[lo + 1], i + 1), L);
    doc_start[i] = s;
    doc_end[i] = e;
    if (is_sep && i - s < a) is_sep[i] = 1;
}

}  // namespace

int launch_doc_bounds(const int32_t *cu_seqlens, int n_docs, int L, int a, int32_t *doc_start, int32_t *doc_end,
                      uint8_t *is_sep, hipStream_t st) {
    ProfScope prof(SEPATTN_K_DOC_BOUNDS, st);
    hipLaunchKernelGGL(doc_bounds_kernel, dim3((L + 255) / 256), dim3(256), 0, st, cu_seqlens, n_docs, L, a,
                       doc_start, doc_end, is_sep);
    return launch_status();
}

}  // namespace sepattn
