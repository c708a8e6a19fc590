// One new token per sequence enters the four-block KV cache (Sec. 3.3 "Framework").  The first a
// tokens of a sequence fill the Initial Cache; every later token is written behind the newest window
// entry (the window region is a ring: entry u sits at index (head + u) mod its capacity) and joins the
// Local Window Cache, whose oldest entry passes to the Past Window Cache once the Local Window holds
// more than w (the window is ordered oldest first, so that hand-over is a change of the two sizes only).  A sequence whose window region [a+s, c) is full is left untouched: the
// compression step has to run first.
//
// One workgroup per sequence; a thread copies 16-byte pieces of the 2 * Hkv rows.  All threads read
// the sizes, then (after a barrier) thread 0 writes the new ones.
#include "decode_common.h"

namespace sepattn {

namespace {

constexpr int kAppendThreads = 256;

__global__ __launch_bounds__(kAppendThreads) void cache_append_kernel(
    sepkv_params p, int row16, const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
    const uint8_t *__restrict__ is_sep_new, uint4 *__restrict__ Kc, uint4 *__restrict__ Vc,
    uint8_t *__restrict__ win_is_sep, int32_t *__restrict__ sizes) {
    const int sq = blockIdx.x;
    int32_t *sz = sizes + SEPKV_SIZES_COLS * sq;
    const CacheMap cm = cache_map(p, sz);
    const int wcap = cm.wcap;
    const int n_init = cm.n_init;
    const int n_past = cm.n_past, n_loc = cm.n_loc;
    const int u = n_past + n_loc;
    __syncthreads();  // every thread has the old sizes before thread 0 replaces them
    int slot;
    if (n_init < p.a)
        slot = n_init;
    else if (u < wcap)
        slot = p.a + p.s + win_index(cm, u);
    else
        return;  // window region full (uniform over the workgroup)
    for (int item = threadIdx.x; item < 2 * p.Hkv * row16; item += kAppendThreads) {
        const int piece = item % row16, kv = (item / row16) % p.Hkv, which = item / (row16 * p.Hkv);
        const uint4 *src = (which ? v_new : k_new) + ((long)sq * p.Hkv + kv) * row16;
        uint4 *dst = (which ? Vc : Kc) + (((long)sq * p.Hkv + kv) * p.c + slot) * (long)row16;
        dst[piece] = src[piece];
    }
    if (threadIdx.x == 0) {
        if (n_init < p.a) {
            sz[0] = n_init + 1;
        } else {
            win_is_sep[(long)sq * wcap + win_index(cm, u)] = is_sep_new[sq] ? 1 : 0;
            const int over = (n_loc + 1 > p.w) ? 1 : 0;
            sz[2] = n_past + over;
            sz[3] = n_loc + 1 - over;
        }
    }
}

}  // namespace

int launch_cache_append(const sepkv_params &p, const void *k_new, const void *v_new, const uint8_t *is_sep_new,
                        void *Kc, void *Vc, uint8_t *win_is_sep, int32_t *sizes, hipStream_t st) {
    const int elem = (p.dtype == SEPATTN_BF16) ? 2 : 4;
    const int row16 = p.d * elem / 16;
    ProfScope prof(SEPATTN_K_CACHE_APPEND, st);
    hipLaunchKernelGGL(cache_append_kernel, dim3(p.S), dim3(kAppendThreads), 0, st, p, row16,
                       static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new), is_sep_new,
                       static_cast<uint4 *>(Kc), static_cast<uint4 *>(Vc), win_is_sep, sizes);
    return launch_status();
}

}  // namespace sepattn
