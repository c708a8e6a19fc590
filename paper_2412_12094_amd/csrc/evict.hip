// Compression step of the four-block KV cache (Sec. 3.3; caption of the streaming-design figure):
// separators of the Past Window move to the Separator Cache, the rest of the Past Window is
// dropped, the Local Window slides to the start of the window region.  In place, bit-exact rows.
//
// Two kernels on the stream:
//   plan: one workgroup per sequence.  Ballot + prefix-sum compaction of the Past-Window flags
//         into a list of kept window slots, the plan numbers (Size_sep, Size_past, Size_local,
//         kept, dropped), then the in-place update of the flag array and of `sizes`.
//   move: one workgroup per (sequence, KV head, K or V).  Three phases separated by barriers:
//         (1) if the Separator Cache overflows, shift its surviving rows down by `dropped`,
//         (2) copy the kept Past-Window rows behind them,
//         (3) slide the Local Window rows to window slot 0.
//         Every phase walks ascending and each chunk of rows is fully read into registers before
//         any of it is written; destinations never lie above their sources, so no row is read
//         after it was overwritten, and one workgroup owns one (sequence, head, tensor), so there
//         is no hazard between workgroups.  The move kernel reads only the plan, never `sizes`
//         or the flags the plan kernel rewrote.
#include "common.h"

namespace sepattn {

namespace {

constexpr int kPlanInts = 8;  // per sequence: Ns, P, Lw, kept, drop, Ns_new
constexpr int kEvictThreads = 256;

__global__ __launch_bounds__(kEvictThreads) void evict_plan_kernel(sepkv_params p,
                                                                   uint8_t *__restrict__ win_is_sep,
                                                                   int32_t *__restrict__ sizes,
                                                                   int32_t *__restrict__ plan,
                                                                   int32_t *__restrict__ kept_list) {
    __shared__ int wave_cnt[kEvictThreads / kWave];
    __shared__ int running;
    int sq = blockIdx.x;
    int wcap = p.c - p.a - p.s;
    int32_t *sz = sizes + 4 * sq;
    int Ns = min(max(sz[1], 0), p.s);
    int P = min(max(sz[2], 0), wcap);
    int Lw = min(max(sz[3], 0), wcap - P);
    uint8_t *fl = win_is_sep + (long)sq * wcap;
    int32_t *kept = kept_list + (long)sq * wcap;
    int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) running = 0;
    __syncthreads();
    // ranks of the flagged Past-Window slots, in slot order
    for (int t0 = 0; t0 < P; t0 += kEvictThreads) {
        int t = t0 + threadIdx.x;
        bool f = (t < P) && fl[t] != 0;
        unsigned long long mask = __ballot(f);
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int before = running;
        for (int w2 = 0; w2 < wave; ++w2) before += wave_cnt[w2];
        if (f) kept[before + __popcll(mask & ((1ull << lane) - 1ull))] = t;
        __syncthreads();
        if (threadIdx.x == 0) {
            int s = running;
            for (int w2 = 0; w2 < kEvictThreads / kWave; ++w2) s += wave_cnt[w2];
            running = s;
        }
        __syncthreads();
    }
    int k = running;
    int total = Ns + k;
    int drop = total > p.s ? total - p.s : 0;
    // slide the Local-Window flags to the front: ascending chunks, read all then write all
    if (P > 0) {
        for (int t0 = 0; t0 < Lw; t0 += kEvictThreads) {
            int t = t0 + threadIdx.x;
            uint8_t v = (t < Lw) ? fl[P + t] : 0;
            __syncthreads();
            if (t < Lw) fl[t] = v;
        }
    }
    if (threadIdx.x == 0) {
        int32_t *pl = plan + (long)sq * kPlanInts;
        pl[0] = Ns;
        pl[1] = P;
        pl[2] = Lw;
        pl[3] = k;
        pl[4] = drop;
        pl[5] = total - drop;
        sz[1] = total - drop;
        sz[2] = 0;
        sz[3] = Lw;
    }
}

// rows are moved as 16-byte pieces; ROW16 = pieces per row
__global__ __launch_bounds__(kEvictThreads) void evict_move_kernel(sepkv_params p, int row16,
                                                                   uint4 *__restrict__ Kc,
                                                                   uint4 *__restrict__ Vc,
                                                                   const int32_t *__restrict__ plan,
                                                                   const int32_t *__restrict__ kept_list) {
    constexpr int kUnroll = 4;
    int blk = blockIdx.x;
    int which = blk & 1;
    int kv = (blk >> 1) % p.Hkv;
    int sq = (blk >> 1) / p.Hkv;
    int wcap = p.c - p.a - p.s;
    const int32_t *pl = plan + (long)sq * kPlanInts;
    int Ns = pl[0], P = pl[1], Lw = pl[2], k = pl[3], drop = pl[4];
    const int32_t *kept = kept_list + (long)sq * wcap;
    uint4 *base = (which ? Vc : Kc) + ((long)sq * p.Hkv + kv) * (long)p.c * row16;
    int rows_per_pass = kEvictThreads / row16;  // row16 divides 256 for d in {64,128}, both dtypes
    int r_in = threadIdx.x / row16, piece = threadIdx.x % row16;

    // (1) surviving old separators: source slot a+drop+t -> a+t, t in [0, Ns-drop)
    int surv = Ns - drop;
    if (drop > 0 && surv > 0) {
        for (int t0 = 0; t0 < surv; t0 += rows_per_pass * kUnroll) {
            uint4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int t = t0 + u * rows_per_pass + r_in;
                if (t < surv) v[u] = base[(long)(p.a + drop + t) * row16 + piece];
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int t = t0 + u * rows_per_pass + r_in;
                if (t < surv) base[(long)(p.a + t) * row16 + piece] = v[u];
            }
        }
    }
    __syncthreads();
    // (2) kept Past-Window rows: combined list index Ns+r -> separator slot Ns+r-drop (if >= 0)
    {
        int first = drop > Ns ? drop - Ns : 0;  // kept entries dropped by an overflow larger than Ns
        for (int r0 = first; r0 < k; r0 += rows_per_pass * kUnroll) {
            uint4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int r = r0 + u * rows_per_pass + r_in;
                if (r < k) v[u] = base[(long)(p.a + p.s + kept[r]) * row16 + piece];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int r = r0 + u * rows_per_pass + r_in;
                if (r < k) base[(long)(p.a + Ns + r - drop) * row16 + piece] = v[u];
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // (3) Local Window: window slot P+t -> t
    if (P > 0) {
        for (int t0 = 0; t0 < Lw; t0 += rows_per_pass * kUnroll) {
            uint4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int t = t0 + u * rows_per_pass + r_in;
                if (t < Lw) v[u] = base[(long)(p.a + p.s + P + t) * row16 + piece];
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                int t = t0 + u * rows_per_pass + r_in;
                if (t < Lw) base[(long)(p.a + p.s + t) * row16 + piece] = v[u];
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

int launch_evict(const sepkv_params &p, void *Kc, void *Vc, uint8_t *win_is_sep, int32_t *sizes,
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
