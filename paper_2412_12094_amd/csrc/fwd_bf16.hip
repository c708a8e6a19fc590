// SepAttention forward, bf16 MFMA (Eq. 1 with the mask of Eq. 2), flash-style with online softmax.
//
// A workgroup (8 waves) owns TP consecutive query positions of GP query heads that share one KV
// head (grouped-query attention: the heads are packed into the row dimension, so K/V tiles and the
// mask are shared).  Each wave owns 32 rows: one head, 32 positions.  The keys a tile can see are
// turned into ONE dense stream,
//     [ initial tokens j < min(a, bs) | separators in [min(a,bs), bs) | band keys bs .. i0+TP-1 ]
// with bs = max(0, i0-n+1) the first key of the first row's neighbour window (Sec. 3.1).  The first
// two parts are visible to every row of the tile (they are older than every window and are initial
// tokens / separators) and are gathered through the compacted separator index list; only band keys
// need the per-element test  j <= i and (i-j < n or j is an initial token or a separator).
//
// Schedule: the two waves that share a SIMD (w and w+4) run half a tile apart ("ping-pong").  Time is
// cut into half-phases separated by workgroup barriers; in every half-phase one wave of each SIMD is
// in its MFMA phase  [O^T += V^T P^T of tile t-1, then S^T = K Q^T of tile t]  while the other is in
// its VALU phase  [mask + online softmax of its tile, global loads of coming tiles].  The matrix
// pipe and the vector ALU of a SIMD are thus busy at the same time without any instruction-level
// interleaving inside a wave.  K tiles live in 3 LDS stages, V tiles and the per-key visibility
// ranges in 4; tiles are filled by direct global->LDS loads (global_load_lds_dwordx4, no staging
// registers) issued about two tiles ahead, unpadded with XOR-swizzled 16-byte chunks (see
// mfma_common.h).  V^T operands are read with ds_read_b64_tr_b16.  A wave
// skips 32-key blocks that lie entirely in its future and drops the mask test on blocks every one
// of its rows sees in full.  The running maximum is only raised when it grows by more than 2^8 (all
// terms carry the same stale maximum, so the result is unchanged), which removes almost every
// rescale of the output accumulators.
#include "common.h"
#include "mfma_common.h"
#include "key_stream.h"

// Phase timing for tuning (compile with -DSEPATTN_X_TIMING; never defined in the product build)
#ifdef SEPATTN_X_TIMING
__device__ unsigned long long g_dbg[8 * 8 * 2048];
extern "C" int sepattn_debug_read(unsigned long long *host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg), sizeof(unsigned long long) * n);
}
#define TICK(k)                              \
    {                                        \
        unsigned long long now_ = clock64(); \
        tacc[k] += now_ - tlast;             \
        tlast = now_;                        \
    }
#else
#define TICK(k)
#endif

namespace sepattn {

namespace {

constexpr float kRescaleThreshold = 8.f;  // log2 units

template <int D, int GP>
__global__ __launch_bounds__(512, 2) void fwd_bf16_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ O, float *__restrict__ LSE) {
    constexpr int NW = 8;
    constexpr int TP = 32 * NW / GP;  // query positions per workgroup
    constexpr int CH = D / 8;         // 16-byte chunks per row
    constexpr int RPL = 64 / CH;      // rows covered by one wave-wide 1 KB load
    constexpr int LOADS = kBN / (RPL * NW);  // wave-wide loads per wave per tensor per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    constexpr int KST = 3, VST = 4;  // LDS stages of K, and of V and the visibility ranges
    constexpr int TILE = kBN * D;    // elements per LDS tile (unpadded, XOR-swizzled chunks)
    static_assert(LOADS >= 1 && LOADS * RPL * NW == kBN, "tile must divide among the waves");

    __shared__ __attribute__((aligned(1024))) uint16_t Ks[KST][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t Vs[VST][TILE];
    __shared__ __attribute__((aligned(16))) int lo_s[VST][kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[VST][kBN];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps branches scalar
    const int grp = wave >> 2;                                  // waves w and w+4 share a SIMD
    const int qi = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv, groups = G / GP;
    const int n_pos_tiles = (p.L + TP - 1) / TP;
    const TileGroup tg = xcd_tile_group(blockIdx.x, n_pos_tiles, p.B * p.Hkv * groups);
    const int tile = n_pos_tiles - 1 - tg.rank;  // late tiles carry more separators: start them first
    const int i0 = tile * TP;
    int y = tg.group;
    const int hg = y % groups;
    const int kv = (y / groups) % p.Hkv;
    const int b = y / (groups * p.Hkv);
    const int head = kv * G + hg * GP + (wave % GP);
    const int pw = i0 + 32 * (wave / GP);  // first position of this wave
    const int iq = pw + qi;                // this lane's query position

    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const uint16_t *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const uint16_t *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;

    const Stream st = make_stream(p, prefix, i0, TP);
    const int n_tiles = (st.n_total + kBN - 1) / kBN;

    // this wave's queries as B operands
    bf16x8 qreg[KSTEPS];
    {
        const uint16_t *qrow = Q + (((long)b * p.Hq + head) * p.L + min(iq, p.L - 1)) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
            qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qrow + ks * 16 + 8 * hh));
    }
    const float sl2 = p.scale * kLog2e_f;

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // m_run in the log2 domain (scores times scale*log2e)
    float alpha_pending = 1.f;             // rescale of oacc decided in a VALU phase, applied in the next MFMA phase

    // ---- tile loads: wave w fills rows (LOADS*w + u)*RPL .. +RPL-1 of a tile with one wave-wide
    // direct global->LDS load per tensor; a lane owns physical chunk lane%CH of row my_row(u)
    const int my_pc = lane % CH, my_sub = lane / CH;
    int raw0[LOADS], raw1[LOADS];  // meta stage: idx entry or prefix[j], and prefix[j+1]
    int vm_issued = 0;             // vector-memory instructions issued in the current phase

    auto issue_meta = [&](int t) {
        if (t >= n_tiles) return;
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            int k = t * kBN + (LOADS * wave + u) * RPL + my_sub;
            // both loads are always issued (clamped addresses) so that their count is exact
            bool dense = k < st.n_dense;
            int j = min(max(st.bs + (k - st.n_dense), 0), p.L - 1);
            int e = min(max(st.sep_lo + k - st.n_init, 0), p.cap - 1);
            const int32_t *pa = dense ? idx + e : prefix + j;
            raw0[u] = *pa;
            raw1[u] = prefix[j + 1];
        });
        vm_issued += 2 * LOADS;
    };
    auto issue_rows = [&](int t) {
        if (t >= n_tiles) return;
        const int ks_ = t % KST, vs_ = t % VST;
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            const int r = (LOADS * wave + u) * RPL + my_sub;  // row of the tile
            const int k = t * kBN + r;
            int j, lo, hi;
            if (k >= st.n_total) {  // padding of the last tile: never visible, any valid row
                j = 0;
                lo = kIntMax;
                hi = -1;
            } else if (k < st.n_init) {
                j = k;
                lo = j;
                hi = kIntMax;
            } else if (k < st.n_dense) {
                // the clamp keeps a stale list tail (caller broke sep_count <= cap) from faulting
                j = min(max(raw0[u], 0), p.L - 1);
                lo = j;
                hi = kIntMax;
            } else {
                j = st.bs + (k - st.n_dense);
                bool always = (j < p.a) || (raw1[u] != raw0[u]);
                lo = j;
                hi = always ? kIntMax : j + p.n - 1;
            }
            if (my_pc == 0) {
                lo_s[vs_][r] = lo;
                hi_s[vs_][r] = hi;
            }
            const int wave_off = (LOADS * wave + u) * RPL * D;  // elements: 1 KB per wave-wide load
            load_to_lds_16(Kh + (long)j * D + swz_chunk<kSwzRow, D>(my_pc, r) * 8, &Ks[ks_][wave_off]);
            load_to_lds_16(Vh + (long)j * D + swz_chunk<kSwzTr, D>(my_pc, r) * 8, &Vs[vs_][wave_off]);
        });
        vm_issued += 2 * LOADS;
    };
    // all loads older than the ones issued in this phase have landed (they complete in order)
    auto wait_older_loads = [&]() {
        if (vm_issued == 4 * LOADS) {
            if constexpr (LOADS == 1)
                asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else
                asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        vm_issued = 0;
    };

    const int a_row = pi_row(qi);
    f32x16 sacc[2];   // scores of the tile between its MFMA phase and its VALU phase
    bf16x8 pb[2][2];  // probabilities of the tile (bf16, B-operand layout) for the next MFMA phase

    // ---- MFMA phase of tile t: O^T += V^T P^T of tile t-1, then S^T = K Q^T of tile t
    auto mfma_phase = [&](int t) {
        __builtin_amdgcn_s_setprio(1);
        const bool do_pv = t > 0, do_qk = t < n_tiles;
        if (__builtin_amdgcn_ballot_w64(alpha_pending != 1.f) != 0ull) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha_pending;
            alpha_pending = 1.f;
        }
        int pmode[2] = {0, 0}, qmode[2] = {0, 0};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (do_pv) pmode[kb] = block_mode(st, (t - 1) * kBN + kb * 32, pw, p.n);
            if (do_qk) qmode[kb] = block_mode(st, t * kBN + kb * 32, pw, p.n);
        }
        const uint16_t *Vst = Vs[(t + VST - 1) % VST];
        const uint16_t *Kst = Ks[t % KST];
        bf16x8 va[DB], ka[KSTEPS];
        auto read_v = [&](int kb, int stp) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#ifdef SEPATTN_X_NOLDS
                va[db] = qreg[db];
#else
                va[db] = lds_read_a_tr_swz<kSwzTr, D>(Vst, kb * 32 + stp * 16, db * 32, lane);
#endif
        };
        auto read_k = [&](int kb) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
#ifdef SEPATTN_X_NOLDS
                ka[ks] = qreg[ks];
#else
                ka[ks] = lds_read_a_swz<kSwzRow, D>(Kst, kb * 32 + a_row, 2 * ks + hh);
#endif
        };
        auto mfma_pv = [&](int kb, int stp) {
#pragma unroll
            for (int db = 0; db < DB; ++db) oacc[db] = mfma_bf16(va[db], pb[kb][stp], oacc[db]);
        };
        auto mfma_qk = [&](int kb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) sacc[kb] = mfma_bf16(ka[ks], qreg[ks], sacc[kb]);
        };
        // order: K reads of a block are in flight while the PV MFMAs of the same block run
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (qmode[kb]) read_k(kb);
            if (pmode[kb]) {
                read_v(kb, 0);
                mfma_pv(kb, 0);
                read_v(kb, 1);
                mfma_pv(kb, 1);
            }
            if (qmode[kb]) mfma_qk(kb);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // ---- VALU phase of tile t: mask, online softmax, probabilities to bf16
    auto valu_phase = [&](int t) {
        int mode[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) mode[kb] = block_mode(st, t * kBN + kb * 32, pw, p.n);
        if (mode[0] == 0 && mode[1] == 0) return;
        const int vs_ = t % VST;
        float m_loc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (mode[kb] == 0) continue;
#ifndef SEPATTN_X_NOMASK
            if (mode[kb] == 2)
#else
            if (false)
#endif
            {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    int base = kb * 32 + 16 * half + 8 * hh;
                    int4 lo0 = *reinterpret_cast<const int4 *>(&lo_s[vs_][base]);
                    int4 lo1 = *reinterpret_cast<const int4 *>(&lo_s[vs_][base + 4]);
                    int4 hi0 = *reinterpret_cast<const int4 *>(&hi_s[vs_][base]);
                    int4 hi1 = *reinterpret_cast<const int4 *>(&hi_s[vs_][base + 4]);
                    int los[8] = {lo0.x, lo0.y, lo0.z, lo0.w, lo1.x, lo1.y, lo1.z, lo1.w};
                    int his[8] = {hi0.x, hi0.y, hi0.z, hi0.w, hi1.x, hi1.y, hi1.z, hi1.w};
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        bool vis = (los[k] <= iq) & (iq <= his[k]);
                        sacc[kb][8 * half + k] = vis ? sacc[kb][8 * half + k] : -INFINITY;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) m_loc = fmaxf(m_loc, sacc[kb][i]);
        }
        float m_new = fmaxf(m_run, pair_max(m_loc * sl2));
        bool grow = m_new > m_run + kRescaleThreshold;
        if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
            float alpha = grow ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
            m_run = grow ? m_new : m_run;
            l_run *= alpha;
            alpha_pending = alpha;
        }
        const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (mode[kb] == 0) continue;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float pr = __builtin_amdgcn_exp2f(fmaf(sacc[kb][i], sl2, neg_m));
                sacc[kb][i] = pr;
                psum += pr;
            }
            pb[kb][0] = pack_bf16x8(sacc[kb], 0);
            pb[kb][1] = pack_bf16x8(sacc[kb], 8);
        }
        l_run += psum;
    };

    // ---- prologue: tiles 0 and 1 on their way into LDS, index entries of tile 2 in flight
    issue_meta(0);
    issue_rows(0);
    issue_meta(1);
    issue_rows(1);
    issue_meta(2);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    vm_issued = 0;
    __syncthreads();

    // Half-phase f: group 0 runs MFMA(t) at f = 2t and VALU(t) at f = 2t+1; group 1 runs MFMA(t)
    // at f = 2t+1 and VALU(t) at f = 2t+2 (its half-phase 0 only issues loads).  Tile T is read from
    // f = 2T (K) to f = 2T+3 (V); its loads are issued at f = 2T-4 (group 1) and 2T-3 (group 0),
    // when the stages it overwrites (tiles T-3 of K, T-4 of V) were last read at f = 2T-5.  A wave
    // waits for its own loads of tile T at the end of its next VALU phase, before f = 2T.
    // Both groups pass 2*n_tiles+1 barriers.  The two loops are written out separately (rather than one
    // loop over half-phases with a role switch) so that every accumulator has one straight-line life.
#ifdef SEPATTN_X_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tlast = clock64();
#endif
    if (grp == 0) {
        for (int t = 0; t <= n_tiles; ++t) {
            mfma_phase(t);
            TICK(1)
            __syncthreads();
            TICK(4)
            if (t < n_tiles) {
                issue_rows(t + 2);
                issue_meta(t + 3);
                TICK(0)
                valu_phase(t);
                TICK(2)
                wait_older_loads();
                TICK(3)
                __syncthreads();
                TICK(4)
            }
        }
    } else {
        issue_rows(2);
        issue_meta(3);
        wait_older_loads();
        __syncthreads();
        for (int t = 0; t <= n_tiles; ++t) {
            mfma_phase(t);
            TICK(1)
            if (t < n_tiles) {
                __syncthreads();
                TICK(4)
                issue_rows(t + 3);
                issue_meta(t + 4);
                TICK(0)
                valu_phase(t);
                TICK(2)
                wait_older_loads();
                TICK(3)
                __syncthreads();
                TICK(4)
            }
        }
    }
#ifdef SEPATTN_X_TIMING
    if (lane == 0 && blockIdx.x < 2048) {
        tacc[5] = n_tiles;
        for (int k = 0; k < 8; ++k) g_dbg[((long)blockIdx.x * 8 + wave) * 8 + k] = tacc[k];
    }
#endif

    // epilogue: normalise, store O (bf16) and LSE (natural log)
    if (__builtin_amdgcn_ballot_w64(alpha_pending != 1.f) != 0ull) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha_pending;
    }
    float l_tot = pair_sum(l_run);
    float inv = 1.f / l_tot;
    if (iq < p.L) {
        long orow = ((long)b * p.Hq + head) * p.L + iq;
        uint16_t *dst = O + orow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                uint2 v = pack_bf16x4(oacc[db][4 * i4] * inv, oacc[db][4 * i4 + 1] * inv,
                                      oacc[db][4 * i4 + 2] * inv, oacc[db][4 * i4 + 3] * inv);
                *reinterpret_cast<uint2 *>(dst + db * 32 + 8 * i4 + 4 * hh) = v;
            }
        if (hh == 0) LSE[orow] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2_f;
    }
}

template <int D>
int launch_fwd(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const int32_t *sep_idx, const int32_t *sep_prefix, uint16_t *O, float *LSE,
               hipStream_t st) {
    int G = p.Hq / p.Hkv;
    int GP = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    int TP = 32 * 8 / GP;
    dim3 grid(((p.L + TP - 1) / TP) * p.B * p.Hkv * (G / GP)), block(512);
    ProfScope prof(SEPATTN_K_FORWARD, st);
    if (GP == 4)
        hipLaunchKernelGGL((fwd_bf16_kernel<D, 4>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    else if (GP == 2)
        hipLaunchKernelGGL((fwd_bf16_kernel<D, 2>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    else
        hipLaunchKernelGGL((fwd_bf16_kernel<D, 1>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    return launch_status();
}

}  // namespace

size_t forward_bf16_workspace(const sepattn_params &) { return 0; }

int launch_forward_bf16(const sepattn_params &p, const void *Q, const void *K, const void *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, void *O, float *LSE,
                        void *, hipStream_t st) {
    auto q = static_cast<const uint16_t *>(Q), k = static_cast<const uint16_t *>(K),
         v = static_cast<const uint16_t *>(V);
    auto o = static_cast<uint16_t *>(O);
    if (p.d == 64) return launch_fwd<64>(p, q, k, v, sep_idx, sep_prefix, o, LSE, st);
    return launch_fwd<128>(p, q, k, v, sep_idx, sep_prefix, o, LSE, st);
}

}  // namespace sepattn
