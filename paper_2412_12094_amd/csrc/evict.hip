// Compression step of the four-block KV cache (Sec. 3.3; caption of the streaming-design figure):
// separators of the Past Window move to the Separator Cache, the rest of the Past Window is
// dropped, the Local Window becomes the whole window.  In place, bit-exact rows.
//
// Both the Separator Cache and the window region are rings (see decode_common.h), so the step moves
// only what the method says must move: the kept Past-Window rows are appended behind the newest
// separator (overwriting the oldest ones when the Separator Cache is full: first in, first out), and
// the Past Window is dropped by advancing the window's head; no surviving row is shifted.
//
// Two kernels on the stream:
//   plan: one workgroup per sequence.  Ballot + prefix-sum compaction of the Past-Window flags
//         into a list of (source window index) of the kept entries, the plan numbers, then the
//         update of `sizes`.  The window flags stay where they are (they move with the head).
//   move: one workgroup per (sequence, KV head, K or V) copies the kept rows.  Sources (window
//         region) and destinations (separator region) are disjoint, so there is no ordering to
//         respect; the move kernel reads only the plan, never `sizes`.
#include "decode_common.h"

namespace sepattn {

namespace {

constexpr int kPlanInts = 8;  // per sequence: first destination index in the separator ring, rows to copy, first kept entry copied
constexpr int kEvictThreads = 256;

__global__ __launch_bounds__(kEvictThreads) void evict_plan_kernel(sepkv_params p,
                                                                   const uint8_t *__restrict__ win_is_sep,
                                                                   int32_t *__restrict__ sizes,
                                                                   int32_t *__restrict__ plan,
                                                                   int32_t *__restrict__ kept_list) {
    __shared__ int wave_cnt[kEvictThreads / kWave];
    __shared__ int running;
    const int sq = blockIdx.x;
    int32_t *sz = sizes + SEPKV_SIZES_COLS * sq;
    const CacheMap cm = cache_map(p, sz);
    const int wcap = cm.wcap, Ns = cm.n_sep, P = cm.n_past, Lw = cm.n_loc;
    const uint8_t *fl = win_is_sep + (long)sq * wcap;
    int32_t *kept = kept_list + (long)sq * wcap;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) running = 0;
    __syncthreads();
    // the flagged Past-Window entries in age order: their indices into the window region
    for (int t0 = 0; t0 < P; t0 += kEvictThreads) {
        const int t = t0 + threadIdx.x;
        const int wi = win_index(cm, min(t, wcap - 1));
        const bool f = (t < P) && fl[wi] != 0;
        const unsigned long long mask = __ballot(f);
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = running;
        for (int w2 = 0; w2 < wave; ++w2) before += wave_cnt[w2];
        if (f) kept[before + __popcll(mask & ((1ull << lane) - 1ull))] = wi;
        __syncthreads();
        if (threadIdx.x == 0) {
            int s = running;
            for (int w2 = 0; w2 < kEvictThreads / kWave; ++w2) s += wave_cnt[w2];
            running = s;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int k = running;
        const int total = Ns + k;
        const int drop = total > p.s ? total - p.s : 0;  // oldest entries of (old separators ++ kept) that fall out
        const int first = drop > Ns ? drop - Ns : 0;     // kept entries that fall out themselves (more new ones than s)
        int32_t *pl = plan + (long)sq * kPlanInts;
        // kept entry r (first <= r < k) goes to ring index (sep_head + Ns + r) mod s
        pl[0] = p.s > 0 ? (cm.sep_head + Ns + first) % p.s : 0;
        pl[1] = p.s > 0 ? k - first : 0;
        pl[2] = first;
        sz[1] = total - drop;
        sz[2] = 0;
        sz[3] = Lw;
        sz[4] = p.s > 0 ? (cm.sep_head + drop) % p.s : 0;
        sz[5] = (cm.win_head + P) % wcap;
    }
}

// rows are moved as 16-byte pieces; row16 = pieces per row
__global__ __launch_bounds__(kEvictThreads) void evict_move_kernel(sepkv_params p, int row16,
                                                                   uint4 *__restrict__ Kc,
                                                                   uint4 *__restrict__ Vc,
                                                                   const int32_t *__restrict__ plan,
                                                                   const int32_t *__restrict__ kept_list) {
    constexpr int kUnroll = 4;
    const int blk = blockIdx.x;
    const int which = blk & 1;
    const int kv = (blk >> 1) % p.Hkv;
    const int sq = (blk >> 1) / p.Hkv;
    const int wcap = p.c - p.a - p.s;
    const int32_t *pl = plan + (long)sq * kPlanInts;
    const int dst0 = pl[0], n_copy = pl[1], first = pl[2];
    const int32_t *kept = kept_list + (long)sq * wcap + first;
    uint4 *base = (which ? Vc : Kc) + ((long)sq * p.Hkv + kv) * (long)p.c * row16;
    const int rows_per_pass = kEvictThreads / row16;  // row16 divides 256 for d in {64,128}, both dtypes
    const int r_in = threadIdx.x / row16, piece = threadIdx.x % row16;
    for (int r0 = 0; r0 < n_copy; r0 += rows_per_pass * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = r0 + u * rows_per_pass + r_in;
            if (r < n_copy) v[u] = base[(long)(p.a + p.s + kept[r]) * row16 + piece];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int r = r0 + u * rows_per_pass + r_in;
            if (r < n_copy) {
                int t = dst0 + r;
                if (t >= p.s) t -= p.s;
                base[(long)(p.a + t) * row16 + piece] = v[u];
            }
        }
    }
}

}  // namespace

size_t evict_workspace(const sepkv_params &p) {
    size_t wcap = (size_t)(p.c - p.a - p.s);
    return align_up((size_t)p.S * kPlanInts * sizeof(int32_t), 256) +
           align_up((size_t)p.S * wcap * sizeof(int32_t), 256);
}

int launch_evict(const sepkv_params &p, void *Kc, void *Vc, const uint8_t *win_is_sep, int32_t *sizes,
                 void *ws, hipStream_t st) {
    int32_t *plan = static_cast<int32_t *>(ws);
    int32_t *kept = reinterpret_cast<int32_t *>(static_cast<char *>(ws) +
                                                align_up((size_t)p.S * kPlanInts * sizeof(int32_t), 256));
    int elem = (p.dtype == SEPATTN_BF16) ? 2 : 4;
    int row16 = p.d * elem / 16;
    {
        ProfScope prof(SEPATTN_K_EVICT_PLAN, st);
        hipLaunchKernelGGL(evict_plan_kernel, dim3(p.S), dim3(kEvictThreads), 0, st, p, win_is_sep, sizes, plan, kept);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_EVICT_MOVE, st);
    hipLaunchKernelGGL(evict_move_kernel, dim3(p.S * p.Hkv * 2), dim3(kEvictThreads), 0, st, p, row16,
                       (uint4 *)Kc, (uint4 *)Vc, plan, kept);
    return launch_status();
}

}  // namespace sepattn
