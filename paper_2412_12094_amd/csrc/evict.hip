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
//   move:  one workgroup per (sequence, KV head, K or V).  Every workgroup derives the plan of its
//          sequence itself from `sizes` and the Past-Window flags (a count, then a ballot + prefix
//          compaction of the flags into a list of kept window indices in shared memory, a chunk of
//          the Past Window at a time) and copies the kept rows of its head; all row loads of a
//          chunk are in flight together.  Sources (window region) and destinations (separator
//          region) are disjoint, so there is no ordering to respect.  It only reads `sizes`.
//   sizes: one workgroup per sequence counts the kept entries again and writes the new `sizes`
//          row.  It runs after the move kernel (stream order), so no workgroup of the move kernel
//          can see the new values.  The window flags stay where they are (they move with the head).
#include "decode_common.h"

namespace sepattn {

namespace {

constexpr int kEvictThreads = 256;
constexpr int kEvictWaves = kEvictThreads / kWave;
constexpr int kChunk = 4 * kEvictThreads;  // Past-Window entries compacted at a time (four per thread)

// what the compression step does to one sequence, from its counts and the number k of flagged
// Past-Window entries: entry r (first <= r < k, in age order) goes to ring index (dst0 + r - first) mod s
struct EvictPlan {
    int dst0, first, n_sep_new, sep_head_new, win_head_new;
};
__device__ inline EvictPlan evict_plan(const sepkv_params &p, const CacheMap &cm, int k) {
    EvictPlan e;
    const int total = cm.n_sep + k;
    const int drop = total > p.s ? total - p.s : 0;       // oldest entries of (old separators ++ kept) that fall out
    e.first = drop > cm.n_sep ? drop - cm.n_sep : 0;      // kept entries that fall out themselves (more new ones than s)
    e.dst0 = p.s > 0 ? (cm.sep_head + cm.n_sep + e.first) % p.s : 0;
    e.n_sep_new = total - drop;
    e.sep_head_new = p.s > 0 ? (cm.sep_head + drop) % p.s : 0;
    e.win_head_new = (cm.win_head + cm.n_past) % cm.wcap;
    return e;
}

// number of flagged entries among the Past Window's P entries (every thread gets the total)
__device__ inline int count_kept(const CacheMap &cm, const uint8_t *__restrict__ fl, int P, int *wave_cnt) {
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int n = 0;
    for (int t = threadIdx.x; t < P; t += kEvictThreads) n += fl[win_index(cm, t)] != 0;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) n += __shfl_xor(n, off);
    if (lane == 0) wave_cnt[wave] = n;
    __syncthreads();
    int k = 0;
#pragma unroll
    for (int w = 0; w < kEvictWaves; ++w) k += wave_cnt[w];
    __syncthreads();
    return k;
}

// rows are moved as 16-byte pieces; row16 = pieces per row
__global__ __launch_bounds__(kEvictThreads) void evict_move_kernel(sepkv_params p, int row16,
                                                                   uint4 *__restrict__ Kc,
                                                                   uint4 *__restrict__ Vc,
                                                                   const uint8_t *__restrict__ win_is_sep,
                                                                   const int32_t *__restrict__ sizes) {
    constexpr int kUnroll = 8;
    __shared__ int wave_cnt[kEvictWaves];
    __shared__ int32_t kept[kChunk];
    const int blk = blockIdx.x;
    const int which = blk & 1;
    const int kv = (blk >> 1) % p.Hkv;
    const int sq = (blk >> 1) / p.Hkv;
    const CacheMap cm = cache_map(p, sizes + SEPKV_SIZES_COLS * sq);
    const int P = cm.n_past;
    if (p.s <= 0 || P <= 0) return;
    const uint8_t *fl = win_is_sep + (long)sq * cm.wcap;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int k = count_kept(cm, fl, P, wave_cnt);
    const EvictPlan pl = evict_plan(p, cm, k);
    uint4 *base = (which ? Vc : Kc) + ((long)sq * p.Hkv + kv) * (long)p.c * row16;
    const int rows_per_pass = kEvictThreads / row16;  // row16 divides 256 for d in {64,128}, both dtypes
    const int r_in = threadIdx.x / row16, piece = threadIdx.x % row16;
    int rank0 = 0;  // kept entries before the chunk
    for (int c0 = 0; c0 < P; c0 += kChunk) {
        // thread t owns the chunk's entries 4t .. 4t+3 (age order): their flags, the count before them
        int wi[4];
        bool f[4];
        int mine = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int t = c0 + 4 * threadIdx.x + e;
            wi[e] = win_index(cm, min(t, cm.wcap - 1));
            f[e] = t < P && fl[wi[e]] != 0;
            mine += f[e];
        }
        int incl = mine;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int u = __shfl_up(incl, off);
            if (lane >= off) incl += u;
        }
        if (lane == kWave - 1) wave_cnt[wave] = incl;
        __syncthreads();
        int before = incl - mine, in_chunk = 0;
#pragma unroll
        for (int w = 0; w < kEvictWaves; ++w) {
            before += w < wave ? wave_cnt[w] : 0;
            in_chunk += wave_cnt[w];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (f[e]) kept[before++] = wi[e];
        __syncthreads();
        // entries of the chunk with rank (rank0 + r) >= first are copied
        const int skip = max(pl.first - rank0, 0);
        for (int r0 = skip; r0 < in_chunk; r0 += rows_per_pass * kUnroll) {
            uint4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * rows_per_pass + r_in;
                if (r < in_chunk) v[u] = base[(long)(p.a + p.s + kept[r]) * row16 + piece];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int r = r0 + u * rows_per_pass + r_in;
                if (r < in_chunk) {
                    int t = pl.dst0 + (rank0 + r - pl.first);
                    if (t >= p.s) t -= p.s;
                    base[(long)(p.a + t) * row16 + piece] = v[u];
                }
            }
        }
        rank0 += in_chunk;
        __syncthreads();  // the list is rewritten by the next chunk
    }
}

__global__ __launch_bounds__(kEvictThreads) void evict_sizes_kernel(sepkv_params p,
                                                                    const uint8_t *__restrict__ win_is_sep,
                                                                    int32_t *__restrict__ sizes) {
    __shared__ int wave_cnt[kEvictWaves];
    const int sq = blockIdx.x;
    int32_t *sz = sizes + SEPKV_SIZES_COLS * sq;
    const CacheMap cm = cache_map(p, sz);
    const int k = count_kept(cm, win_is_sep + (long)sq * cm.wcap, cm.n_past, wave_cnt);
    if (threadIdx.x == 0) {
        const EvictPlan pl = evict_plan(p, cm, k);
        sz[1] = pl.n_sep_new;
        sz[2] = 0;
        sz[3] = cm.n_loc;
        sz[4] = pl.sep_head_new;
        sz[5] = pl.win_head_new;
    }
}

}  // namespace

// the step needs no scratch memory; the query stays in the interface and answers 0
size_t evict_workspace(const sepkv_params &) { return 0; }

int launch_evict(const sepkv_params &p, void *Kc, void *Vc, const uint8_t *win_is_sep, int32_t *sizes,
                 void *, hipStream_t st) {
    int elem = (p.dtype == SEPATTN_BF16) ? 2 : 4;
    int row16 = p.d * elem / 16;
    {
        ProfScope prof(SEPATTN_K_EVICT_MOVE, st);
        hipLaunchKernelGGL(evict_move_kernel, dim3(p.S * p.Hkv * 2), dim3(kEvictThreads), 0, st, p, row16,
                           (uint4 *)Kc, (uint4 *)Vc, win_is_sep, sizes);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_EVICT_SIZES, st);
    hipLaunchKernelGGL(evict_sizes_kernel, dim3(p.S), dim3(kEvictThreads), 0, st, p, win_is_sep, sizes);
    return launch_status();
}

}  // namespace sepattn
