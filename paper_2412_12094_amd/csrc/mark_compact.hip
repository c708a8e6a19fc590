// Separator marking and compaction (integer kernels).
//
// mark:    is_sep[t] = token_ids[t] in S, S = the caller's separator id set (Sec. 4.1 "Parameter
//          Setting").  One thread per four tokens, the id set travels in the kernel arguments.
// compact: the index form of the separator part of mask M (Eq. 2): ascending separator positions,
//          their count and the exclusive prefix count per sequence.  Two passes over chunks of
//          2048 tokens: (1) per-chunk separator counts, (2) each chunk sums the counts of the
//          chunks before it, ranks its own separators with wave ballots + a block prefix sum over
//          the per-wave counts, and writes prefix / index entries.  No atomics, so the output
//          order is the position order by construction.  Sequences of up to 32768 tokens take
//          one launch: pass (2) then counts the flags of the earlier chunks itself.
// mark + compact in one launch (sequences of up to 8192 tokens): pass (2) reads the token ids, tests
//          them against the id set itself and also writes the marker bitmap; at these sizes each
//          of the two kernels lasts no longer than its launch.
#include "common.h"

namespace sepattn {

__global__ __launch_bounds__(256) void mark_kernel(const int32_t *__restrict__ ids, long n,
                                                   SepIdSet set, uint8_t *__restrict__ out) {
    long t4 = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (t4 >= n) return;
    if (t4 + 4 <= n) {
        int4 v = *reinterpret_cast<const int4 *>(ids + t4);
        unsigned f0 = 0, f1 = 0, f2 = 0, f3 = 0;
        for (int k = 0; k < set.n; ++k) {
            int s = set.ids[k];
            f0 |= (v.x == s);
            f1 |= (v.y == s);
            f2 |= (v.z == s);
            f3 |= (v.w == s);
        }
        *reinterpret_cast<uint32_t *>(out + t4) = f0 | (f1 << 8) | (f2 << 16) | (f3 << 24);
    } else {
        for (long t = t4; t < n; ++t) {
            unsigned f = 0;
            for (int k = 0; k < set.n; ++k) f |= (ids[t] == set.ids[k]);
            out[t] = (uint8_t)f;
        }
    }
}

int launch_mark(const int32_t *token_ids, long n_tokens, const SepIdSet &set, uint8_t *is_sep,
                hipStream_t st) {
    long threads = (n_tokens + 3) / 4;
    unsigned blocks = (unsigned)((threads + 255) / 256);
    ProfScope prof(SEPATTN_K_MARK, st);
    hipLaunchKernelGGL(mark_kernel, dim3(blocks), dim3(256), 0, st, token_ids, n_tokens, set, is_sep);
    return launch_status();
}

// Fixed-interval variant ("FixLLM", the appendix on the fixed-interval variant): one token in every
// `delta` is marked instead of the separators: position j of every sequence iff j % delta == phase.
__global__ __launch_bounds__(256) void mark_interval_kernel(int L, long n, int delta, int phase,
                                                            uint8_t *__restrict__ out) {
    const long t4 = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (t4 >= n) return;
    int r = (int)((t4 % L) % delta);  // residue of the first of this thread's four positions
    int j = (int)(t4 % L);
    unsigned f[4];
    for (int k = 0; k < 4; ++k) {
        f[k] = (r == phase);
        ++j;
        r = (r + 1 == delta) ? 0 : r + 1;
        if (j == L) {  // next sequence
            j = 0;
            r = 0;
        }
    }
    if (t4 + 4 <= n) {
        *reinterpret_cast<uint32_t *>(out + t4) = f[0] | (f[1] << 8) | (f[2] << 16) | (f[3] << 24);
    } else {
        for (int k = 0; t4 + k < n; ++k) out[t4 + k] = (uint8_t)f[k];
    }
}

int launch_mark_interval(int B, int L, int delta, int phase, uint8_t *is_sep, hipStream_t st) {
    const long n = (long)B * L, threads = (n + 3) / 4;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    ProfScope prof(SEPATTN_K_MARK_INTERVAL, st);
    hipLaunchKernelGGL(mark_interval_kernel, dim3(blocks), dim3(256), 0, st, L, n, delta, phase, is_sep);
    return launch_status();
}

// ---- compaction --------------------------------------------------------------------------------
constexpr int kCompactThreads = 256;
constexpr int kCompactSingleLaunch = 32768;  // longest sequence compacted with one launch
constexpr int kMarkCompactSingleLaunch = 8192;  // longest sequence marked and compacted with one launch
constexpr int kCompactIters = kCompactChunk / kCompactThreads;  // 8 ballots per wave per chunk
constexpr int kCompactWaves = kCompactThreads / kWave;

// pass 1: chunk_counts[b, chunk] = number of separators in the chunk
__global__ __launch_bounds__(kCompactThreads) void compact_count_kernel(
    const uint8_t *__restrict__ is_sep, int L, int n_chunks, int32_t *__restrict__ chunk_counts) {
    __shared__ int wave_cnt[kCompactWaves];
    int b = blockIdx.y, chunk = blockIdx.x;
    const uint8_t *row = is_sep + (long)b * L;
    int base = chunk * kCompactChunk;
    int cnt = 0;
    for (int it = 0; it < kCompactIters; ++it) {
        int j = base + it * kCompactThreads + threadIdx.x;
        bool f = (j < L) && row[j] != 0;
        cnt += __popcll(__ballot(f));
    }
    int wave = threadIdx.x / kWave;
    if (threadIdx.x % kWave == 0) wave_cnt[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int w = 0; w < kCompactWaves; ++w) s += wave_cnt[w];
        chunk_counts[(long)b * n_chunks + chunk] = s;
    }
}

__device__ inline bool in_id_set(int v, const SepIdSet &set) {
    unsigned f = 0;
    for (int k = 0; k < set.n; ++k) f |= (v == set.ids[k]);
    return f != 0;
}

// pass 2: ranks and writes.  FUSED: the flags are not read from is_sep but formed from the token ids
// (and written to marks_out for the chunk's own positions); chunk_counts is nullptr then.
template <bool FUSED>
__global__ __launch_bounds__(kCompactThreads) void compact_write_kernel(
    const uint8_t *__restrict__ is_sep, const int32_t *__restrict__ token_ids, SepIdSet set,
    uint8_t *__restrict__ marks_out, int L, int n_chunks, const int32_t *__restrict__ chunk_counts,
    int32_t *__restrict__ sep_idx, int cap, int32_t *__restrict__ sep_count,
    int32_t *__restrict__ sep_prefix) {
    __shared__ int part[kCompactIters * kCompactWaves];  // count of (iteration, wave) groups
    __shared__ int base_s;
    int b = blockIdx.y, chunk = blockIdx.x;
    const uint8_t *row = FUSED ? nullptr : is_sep + (long)b * L;
    const int32_t *ids_row = FUSED ? token_ids + (long)b * L : nullptr;
    int base = chunk * kCompactChunk;
    int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;

    // separators in earlier chunks of this sequence: from the counts of pass 1, or (short sequences,
    // single launch) counted here from the flags themselves
    if (chunk_counts != nullptr) {
        if (wave == 0) {
            int s = 0;
            for (int c = lane; c < chunk; c += kWave) s += chunk_counts[(long)b * n_chunks + c];
            for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
            if (lane == 0) base_s = s;
        }
    } else {
        __shared__ int early[kCompactWaves];
        int s = 0;
        if constexpr (FUSED) {
            // at most three chunks lie in front (8192 tokens per launch).  All loads of a thread are
            // requested first; the id set is walked in the OUTER loop (one scalar load per id, not
            // one per id and token), a token's matches are collected as bits and counted once, so
            // that an id given twice does not count twice.
            constexpr int kEarly = (kMarkCompactSingleLaunch - kCompactChunk) / (kCompactThreads * 4);
            if ((reinterpret_cast<uintptr_t>(ids_row) & 15u) == 0) {  // base is a multiple of 4
                int4 v[kEarly];
                uint32_t there = 0, hit = 0;
#pragma unroll
                for (int q = 0; q < kEarly; ++q) {
                    const int j = (q * kCompactThreads + (int)threadIdx.x) * 4;
                    v[q] = j < base ? *reinterpret_cast<const int4 *>(ids_row + j) : int4{0, 0, 0, 0};
                    there |= (j < base ? 0xFu : 0u) << (4 * q);
                }
                for (int k = 0; k < set.n; ++k) {
                    const int sid = set.ids[k];
#pragma unroll
                    for (int q = 0; q < kEarly; ++q)
                        hit |= ((uint32_t)(v[q].x == sid) | ((uint32_t)(v[q].y == sid) << 1) | ((uint32_t)(v[q].z == sid) << 2) |
                                ((uint32_t)(v[q].w == sid) << 3))
                               << (4 * q);
                }
                s = __popc(hit & there);
            } else {
                for (int j = threadIdx.x; j < base; j += kCompactThreads) s += in_id_set(ids_row[j], set);
            }
        } else if ((reinterpret_cast<uintptr_t>(row) & 3u) == 0) {  // base is a multiple of 4
            for (int j = threadIdx.x * 4; j < base; j += kCompactThreads * 4) {
                const uint32_t w = *reinterpret_cast<const uint32_t *>(row + j);
                // one bit per non-zero byte
                s += __popc((((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u);
            }
        } else {
            for (int j = threadIdx.x; j < base; j += kCompactThreads) s += row[j] != 0;
        }
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0) early[wave] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            int t = 0;
            for (int w2 = 0; w2 < kCompactWaves; ++w2) t += early[w2];
            base_s = t;
        }
    }
    unsigned long long lt_mask = (1ull << lane) - 1ull;
    bool flag[kCompactIters];
    int rank_in_wave[kCompactIters];
    uint32_t own_hit = 0;
    if constexpr (FUSED) {
        int own_id[kCompactIters];
#pragma unroll
        for (int it = 0; it < kCompactIters; ++it) own_id[it] = ids_row[min(base + it * kCompactThreads + (int)threadIdx.x, L - 1)];
        for (int k = 0; k < set.n; ++k) {
            const int sid = set.ids[k];
#pragma unroll
            for (int it = 0; it < kCompactIters; ++it) own_hit |= (uint32_t)(own_id[it] == sid) << it;
        }
    }
#pragma unroll
    for (int it = 0; it < kCompactIters; ++it) {
        int j = base + it * kCompactThreads + threadIdx.x;
        if constexpr (FUSED) {
            flag[it] = (j < L) && ((own_hit >> it) & 1u);
            if (j < L) marks_out[(long)b * L + j] = flag[it] ? 1 : 0;
        } else {
            flag[it] = (j < L) && row[j] != 0;
        }
        unsigned long long m = __ballot(flag[it]);
        rank_in_wave[it] = __popcll(m & lt_mask);
        if (lane == 0) part[it * kCompactWaves + wave] = __popcll(m);
    }
    __syncthreads();
    // exclusive prefix over the 32 (iteration, wave) groups, in position order, by wave 0
    if (wave == 0) {
        int v = (lane < kCompactIters * kCompactWaves) ? part[lane] : 0;
        int incl = v;
        for (int off = 1; off < kCompactIters * kCompactWaves; off <<= 1) {
            int t = __shfl_up(incl, off);
            if (lane >= off) incl += t;
        }
        if (lane < kCompactIters * kCompactWaves) part[lane] = incl - v;
    }
    __syncthreads();
    int chunk_base = base_s;
    for (int it = 0; it < kCompactIters; ++it) {
        int j = base + it * kCompactThreads + threadIdx.x;
        if (j < L) {
            int r = chunk_base + part[it * kCompactWaves + wave] + rank_in_wave[it];
            if (sep_prefix) sep_prefix[(long)b * (L + 1) + j] = r;
            if (flag[it] && r < cap) sep_idx[(long)b * cap + r] = j;
            if (j == L - 1) {
                int total = r + (flag[it] ? 1 : 0);
                if (sep_prefix) sep_prefix[(long)b * (L + 1) + L] = total;
                sep_count[b] = total;
            }
        }
    }
}

int launch_compact(const uint8_t *is_sep, int B, int L, int32_t *sep_idx, int cap,
                   int32_t *sep_count, int32_t *sep_prefix, int32_t *chunk_counts, hipStream_t st) {
    int n_chunks = (L + kCompactChunk - 1) / kCompactChunk;
    dim3 grid(n_chunks, B);
    // Up to kCompactSingleLaunch positions a workgroup counts the separators in front of its chunk
    // itself (at most that many flag bytes, read once more): one launch instead of two, which matters
    // because at these sizes the kernels last no longer than their launch.
    const bool single = L <= kCompactSingleLaunch;
    if (!single) {
        ProfScope prof(SEPATTN_K_COMPACT_COUNT, st);
        hipLaunchKernelGGL(compact_count_kernel, grid, dim3(kCompactThreads), 0, st, is_sep, L, n_chunks,
                           chunk_counts);
        if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    }
    ProfScope prof(SEPATTN_K_COMPACT_WRITE, st);
    hipLaunchKernelGGL(compact_write_kernel<false>, grid, dim3(kCompactThreads), 0, st, is_sep, nullptr, SepIdSet{},
                       nullptr, L, n_chunks, single ? nullptr : chunk_counts, sep_idx, cap, sep_count, sep_prefix);
    return launch_status();
}

// marking and compaction together: one launch for sequences of up to kMarkCompactSingleLaunch tokens
// (a workgroup then tests the ids in front of its chunk once more to count them), the separate
// kernels beyond
int launch_mark_compact(const int32_t *token_ids, int B, int L, const SepIdSet &set, uint8_t *is_sep,
                        int32_t *sep_idx, int cap, int32_t *sep_count, int32_t *sep_prefix,
                        int32_t *chunk_counts, hipStream_t st) {
    if (L > kMarkCompactSingleLaunch) {
        int rc = launch_mark(token_ids, (long)B * L, set, is_sep, st);
        if (rc != SEPATTN_OK) return rc;
        return launch_compact(is_sep, B, L, sep_idx, cap, sep_count, sep_prefix, chunk_counts, st);
    }
    int n_chunks = (L + kCompactChunk - 1) / kCompactChunk;
    ProfScope prof(SEPATTN_K_MARK_COMPACT, st);
    hipLaunchKernelGGL(compact_write_kernel<true>, dim3(n_chunks, B), dim3(kCompactThreads), 0, st, nullptr, token_ids,
                       set, is_sep, L, n_chunks, nullptr, sep_idx, cap, sep_count, sep_prefix);
    return launch_status();
}

}  // namespace sepattn
