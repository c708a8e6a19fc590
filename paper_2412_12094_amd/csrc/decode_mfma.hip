// Single-query attention over the four-block KV cache (Sec. 3.2 "Generation", Sec. 3.3), bf16,
// as a stream through the matrix cores.
//
// Every valid cache entry is visible, so this is Eq. 1 with one query row per head and M = 1.  The
// work is HBM-bound: K and V are read once (2 * entries * d * 2 bytes per (sequence, KV head)) and
// there are only a few flops per byte.  The kernel is therefore built around keeping many bytes in
// flight per compute unit and spending as few vector-ALU instructions per byte as possible:
//   - a workgroup (4 waves) owns one (sequence, KV head) and one of `nsplit` contiguous slices of
//     its valid entries; the slice is cut into blocks of 32 entries dealt round-robin to the waves;
//   - each wave has a private ring of two LDS stages (32 rows of K and of V each) filled with direct
//     global->LDS loads, 64 lanes x 16 bytes = whole cache rows per instruction; a wave only ever
//     waits on its own loads (s_waitcnt vmcnt), so there is no workgroup barrier in the loop and
//     a stage is refilled as soon as its rows sit in registers, so nearly two stages per wave
//     (32 KB at d = 128) are in flight at any time;
//   - the contractions run on v_mfma_f32_32x32x16_bf16 with the 32 cache rows as the A operand and
//     all query heads of the KV head (grouped-query attention) as columns of the B operand: the
//     scores of a block cost 8 matrix instructions instead of 32 x 128 multiply-adds per head, and
//     bf16 data never has to be widened on the vector ALU.  The unused columns hold zero queries;
//   - online softmax per lane pair as in the training forward; the four waves' (max, sum, output)
//     states are merged through LDS at the end.  With nsplit == 1 the workgroup writes the final
//     output, else a partial record that decode_merge_kernel combines.
//
// Positions within the cache (Sec. 3.3 "Positional Encoding", Sec. 4.6): with ROPE the cache holds
// keys without position encoding and the kernel turns every key row by its position among the valid
// entries (oldest = 0) and the query by the newest entry's position, on the way from LDS to the
// matrix cores.  A lane always reads the same row of a block and the same 2 x 8-element pieces of
// it, and dimension i pairs with i + D/2, i.e. with the same element of another piece the lane
// holds, so the rotation needs no exchange between lanes: a lane keeps cos / sin of its row's
// position for its D/4 frequencies in registers (read once from the caller's table) and advances
// them from one of its blocks to the next (128 positions on) with the angle-sum formulas.
#include "common.h"
#include "mfma_common.h"
#include "decode_common.h"


namespace sepattn {

namespace {

constexpr int kDmWaves = 4;
constexpr int kDmThreads = 64 * kDmWaves;
constexpr int kDmRows = 32;  // cache rows per stage
constexpr int kDmStages = 2;

__device__ inline f32x8 widen(bf16x8 v) { return __builtin_convertvector(v, f32x8); }
__device__ inline bf16x8 narrow(f32x8 v) { return __builtin_convertvector(v, bf16x8); }  // round to nearest even

// rope: [n_pos][2][D/2] fp32, cos then sin of position * base^(-2i/D); only read with ROPE
template <int D, bool ROPE>
__global__ __launch_bounds__(kDmThreads, 1) void decode_mfma_kernel(
    sepkv_params p, int G, const uint16_t *__restrict__ q, const uint16_t *__restrict__ Kc,
    const uint16_t *__restrict__ Vc, const int32_t *__restrict__ sizes, const float *__restrict__ rope, int n_pos,
    float *__restrict__ part, uint16_t *__restrict__ out, float *__restrict__ lse) {
    constexpr int CH = D / 8;          // 16-byte chunks per row
    constexpr int RPL = 64 / CH;       // rows covered by one wave-wide 1 KB load
    constexpr int NLD = kDmRows / RPL; // wave-wide loads per tensor per stage
    constexpr int KSTEPS = D / 16;
    constexpr int KS2 = KSTEPS / 2;    // a lane's piece ks (dimensions 16 ks + 8 hh ..) pairs with piece ks + KS2
    constexpr int DB = D / 32;
    constexpr int TILE = kDmRows * D;  // elements per stage and tensor
    constexpr int PF = D + 2;          // partial record: max (log2 domain), sum, D unnormalised outputs

    // [0]: K stages, [1]: V stages; the merge records overlay the rings once they are drained
    __shared__ __attribute__((aligned(1024))) uint16_t smem[2][kDmWaves][kDmStages][TILE];
    auto &Ks = smem[0];
    auto &Vs = smem[1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;  // column of the B operand = query head of the group
    // grid (nsplit, Hkv, S): no integer division on the way to the first load
    const int nsplit = gridDim.x, split = blockIdx.x, kv = blockIdx.y, sq = blockIdx.z;
    const int h0 = kv * G;

    const uint16_t *Kh = Kc + ((long)sq * p.Hkv + kv) * (long)p.c * D;
    const uint16_t *Vh = Vc + ((long)sq * p.Hkv + kv) * (long)p.c * D;

    // the query fetch is independent of `sizes`; it is issued first and consumed only after the first
    // two stages are on their way, so that the kernel pays one memory latency before streaming, not two
    u32x4 qraw[KSTEPS];
    {
        const uint16_t *qrow = q + ((long)sq * p.Hq + h0 + min(col, G - 1)) * D;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) qraw[ks] = *reinterpret_cast<const u32x4 *>(qrow + ks * 16 + 8 * hh);
    }

    const CacheMap cm = cache_map(p, sizes + SEPKV_SIZES_COLS * sq);
    const int nv = cm.n_init + cm.n_sep + cm.n_past + cm.n_loc;
    int per = (nv + nsplit - 1) / nsplit;
    per = (per + kDmRows - 1) / kDmRows * kDmRows;
    const int e0 = min(split * per, nv), e1 = min(nv, e0 + per);
    const int n_blocks = (e1 - e0 + kDmRows - 1) / kDmRows;
    const int n_my = (n_blocks > wave) ? (n_blocks - wave + kDmWaves - 1) / kDmWaves : 0;

    const float sl2 = p.scale * kLog2e_f;

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int my_pc = lane % CH, my_sub = lane / CH;
    // stage k of this wave <- block wave + 4k of the slice; entries past the slice end are clamped
    // to its last entry (their scores are masked)
    auto issue_stage = [&](int k) {
        const int stg = k % kDmStages;
        const int eb = e0 + (wave + kDmWaves * k) * kDmRows;
        static_for<NLD>([&](auto U) {
            constexpr int u = U;
            const int r = u * RPL + my_sub;
            const int sl = decode_slot_of(cm, min(eb + r, e1 - 1));
            const uint32_t row_off = (uint32_t)sl * (uint32_t)(D * 2);  // a cache of one (sequence, head) is < 4 GB
            // every cache row is read exactly once per call: the non-temporal hint keeps the stream from
            // displacing itself in the caches (measured: 79 -> 71 us at 32 x 8 caches of 3332 entries)
            dma_to_lds_16_nt(Kh, row_off + swz_chunk<kSwzRow, D>(my_pc, r) * 16, lds_addr(&Ks[wave][stg][u * RPL * D]));
            dma_to_lds_16_nt(Vh, row_off + swz_chunk<kSwzTr, D>(my_pc, r) * 16, lds_addr(&Vs[wave][stg][u * RPL * D]));
        });
    };
    // the loads of a stage are 2*NLD instructions; they complete in issue order
    auto wait_older_stage = [&](bool newer_in_flight) {
        if (!newer_in_flight) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else if constexpr (2 * NLD == 16) {
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        } else {
            static_assert(2 * NLD == 8 || 2 * NLD == 16, "wait counts are written for d = 64 and 128");
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        }
    };

    const int a_row = pi_row(col);
    if (n_my > 0) issue_stage(0);
    if (n_my > 1) issue_stage(1);
    // queries as B operands: column = head of the group, zero beyond G
    bf16x8 qreg[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) qreg[ks] = as_bf16x8(col < G ? qraw[ks] : u32x4{0u, 0u, 0u, 0u});

    // cos / sin of a table row for this lane's frequencies 16 ks + 8 hh + (0..7), ks < KS2
    f32x8 rc[KS2], rs[KS2];  // of this lane's row in its next block
    f32x8 tc[KS2], ts[KS2];  // of the distance between two of its blocks
    auto table_row = [&](int pos, f32x8(&co)[KS2], f32x8(&si)[KS2]) {
        const float *row = rope + (long)min(max(pos, 0), n_pos - 1) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) {
            const f32x4 c0 = *reinterpret_cast<const f32x4 *>(row + 16 * ks), c1 = *reinterpret_cast<const f32x4 *>(row + 16 * ks + 4);
            const f32x4 s0 = *reinterpret_cast<const f32x4 *>(row + D / 2 + 16 * ks), s1 = *reinterpret_cast<const f32x4 *>(row + D / 2 + 16 * ks + 4);
            co[ks] = f32x8{c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
            si[ks] = f32x8{s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
        }
    };
    // (x, y) -> (x cos - y sin, y cos + x sin) on a pair of pieces
    auto turn = [&](bf16x8 &lo, bf16x8 &hi, const f32x8 &co, const f32x8 &si) {
        const f32x8 x = widen(lo), y = widen(hi);
        lo = narrow(x * co - y * si);
        hi = narrow(y * co + x * si);
    };
    if constexpr (ROPE) {
        table_row(nv - 1, rc, rs);  // the query is the newest entry's token
#pragma unroll
        for (int ks = 0; ks < KS2; ++ks) turn(qreg[ks], qreg[ks + KS2], rc[ks], rs[ks]);
        table_row(e0 + wave * kDmRows + a_row, rc, rs);
        table_row(kDmWaves * kDmRows, tc, ts);
    }

    for (int k = 0; k < n_my; ++k) {
        wait_older_stage(k + 1 < n_my);
        const uint16_t *Kst = Ks[wave][k % kDmStages];
        const uint16_t *Vst = Vs[wave][k % kDmStages];
        const int n_valid = e1 - (e0 + (wave + kDmWaves * k) * kDmRows);  // >= 1; >= 32 except in the last block

        // S^T = K q^T
        f32x16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
        {
            bf16x8 ka[KSTEPS];
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) ka[ks] = lds_read_a_swz<kSwzRow, D>(Kst, a_row, 2 * ks + hh);
            if constexpr (ROPE) {
#pragma unroll
                for (int ks = 0; ks < KS2; ++ks) turn(ka[ks], ka[ks + KS2], rc[ks], rs[ks]);
            }
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) sacc = mfma_bf16(ka[ks], qreg[ks], sacc);
        }
        // V^T fragments are requested before the softmax arithmetic that hides their latency
        bf16x8 va[2][DB];
#pragma unroll
        for (int stp = 0; stp < 2; ++stp)
#pragma unroll
            for (int db = 0; db < DB; ++db)
                va[stp][db] = lds_read_a_tr_swz<kSwzTr, D>(Vst, stp * 16, db * 32, lane);
        // both tiles of the stage now sit in registers (the score MFMAs above consumed K): refill the
        // stage at once, so that the wave has two stages in flight for all but the first few hundred
        // cycles of a block
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (k + kDmStages < n_my) issue_stage(k + kDmStages);
        if constexpr (ROPE) {
            // the lane's row of its next block lies kDmWaves * kDmRows positions further on
#pragma unroll
            for (int ks = 0; ks < KS2; ++ks) {
                const f32x8 c_old = rc[ks];
                rc[ks] = c_old * tc[ks] - rs[ks] * ts[ks];
                rs[ks] = rs[ks] * tc[ks] + c_old * ts[ks];
            }
        }

        if (n_valid < kDmRows) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (rho_row(hh, i) >= n_valid) sacc[i] = -INFINITY;
        }
        float m_loc = sacc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) m_loc = fmaxf(m_loc, sacc[i]);
        // row 0 of every block is valid, so the new maximum is finite
        const float m_new = fmaxf(m_run, pair_max(m_loc * sl2));
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pr = __builtin_amdgcn_exp2f(fmaf(sacc[i], sl2, -m_new));
            sacc[i] = pr;
            psum += pr;
        }
        l_run = l_run * alpha + psum;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }
        const bf16x8 pb0 = pack_bf16x8(sacc, 0), pb1 = pack_bf16x8(sacc, 8);
        // O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = mfma_bf16(va[0][db], pb0, oacc[db]);
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = mfma_bf16(va[1][db], pb1, oacc[db]);

    }

    // ---- merge the four waves' states through LDS (the rings are no longer in use)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    float *red = reinterpret_cast<float *>(&smem[0][0][0][0]);  // [G][kDmWaves][PF]
    static_assert(sizeof(smem) >= 32 * kDmWaves * PF * sizeof(float), "merge records must fit in the rings");
    const float l_tot = pair_sum(l_run);
    if (col < G) {
        float *r = red + (col * kDmWaves + wave) * PF;
        if (hh == 0) {
            r[0] = m_run;
            r[1] = l_tot;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = {oacc[db][4 * i4], oacc[db][4 * i4 + 1], oacc[db][4 * i4 + 2], oacc[db][4 * i4 + 3]};
                *reinterpret_cast<f32x4 *>(r + 2 + db * 32 + 8 * i4 + 4 * hh) = v;
            }
    }
    __syncthreads();
    for (int item = tid; item < G * D; item += kDmThreads) {
        const int g = item / D, c = item % D;
        const float *r = red + g * kDmWaves * PF;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDmWaves; ++w) M = fmaxf(M, r[w * PF]);
        float lsum = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kDmWaves; ++w) {
            const float ms = r[w * PF];
            const float wgt = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - M);
            lsum = fmaf(wgt, r[w * PF + 1], lsum);
            o = fmaf(wgt, r[w * PF + 2 + c], o);
        }
        const long sh = (long)sq * p.Hq + h0 + g;
        if (nsplit == 1) {
            const float val = (lsum > 0.f) ? o / lsum : 0.f;
            out[sh * D + c] = decode_f32_to_bf16(val);
            if (lse && c == 0) lse[sh] = (lsum > 0.f) ? (M + __builtin_amdgcn_logf(lsum)) * kLn2_f : -INFINITY;
        } else {
            float *dst = part + (sh * nsplit + split) * PF;
            dst[2 + c] = o;
            if (c == 0) {
                dst[0] = M;
                dst[1] = lsum;
            }
        }
    }
}

}  // namespace

bool decode_mfma_applicable(const sepkv_params &p) {
    return p.dtype == SEPATTN_BF16 && (p.d == 64 || p.d == 128) && p.Hq / p.Hkv <= 32;
}

int decode_mfma_nsplit(const sepkv_params &p) {
    // one workgroup per compute unit keeps two stages per wave in flight; aim at >= 256 workgroups,
    // but never cut a cache into slices of fewer than 256 entries
    const long pairs = (long)p.S * p.Hkv;
    long want = (256 + pairs - 1) / pairs;
    const long max_by_rows = (p.c + 255) / 256;
    if (want > max_by_rows) want = max_by_rows;
    return (int)(want < 1 ? 1 : (want > 64 ? 64 : want));
}

int launch_decode_mfma(const sepkv_params &p, int nsplit, const uint16_t *q, const uint16_t *Kc, const uint16_t *Vc,
                       const int32_t *sizes, const float *rope, int n_pos, uint16_t *out, float *lse, float *part,
                       hipStream_t st) {
    if (p.Hkv > 65535 || p.S > 65535) return SEPATTN_ERR_SHAPE;
    const dim3 grid(nsplit, p.Hkv, p.S), block(kDmThreads);
    const int G = p.Hq / p.Hkv;
    ProfScope prof(SEPATTN_K_DECODE_SPLIT, st);
    if (p.d == 64 && rope)
        hipLaunchKernelGGL((decode_mfma_kernel<64, true>), grid, block, 0, st, p, G, q, Kc, Vc, sizes, rope, n_pos, part, out, lse);
    else if (p.d == 64)
        hipLaunchKernelGGL((decode_mfma_kernel<64, false>), grid, block, 0, st, p, G, q, Kc, Vc, sizes, rope, n_pos, part, out, lse);
    else if (rope)
        hipLaunchKernelGGL((decode_mfma_kernel<128, true>), grid, block, 0, st, p, G, q, Kc, Vc, sizes, rope, n_pos, part, out, lse);
    else
        hipLaunchKernelGGL((decode_mfma_kernel<128, false>), grid, block, 0, st, p, G, q, Kc, Vc, sizes, rope, n_pos, part, out, lse);
    return launch_status();
}

}  // namespace sepattn
