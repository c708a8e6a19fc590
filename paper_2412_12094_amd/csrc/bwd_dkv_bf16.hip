// SepAttention backward, dK and dV (bf16 MFMA): the analytic gradient of Eq. 1 under the mask of Eq. 2,
//   dV_j = sum_i P_ij dO_i,   dK_j = scale sum_i dS_ij Q_i,   dS_ij = P_ij (<dO_i, V_j> - D_i),
//   P_ij = exp(scale <Q_i, K_j> - LSE_i),  summed over the query heads of the KV head.
//
// The visible pairs split into band pairs (i-j < n) and far pairs (i-j >= n, j an initial token or a
// separator, Sec. 3.1).
//   dkv_kernel<far>:  far pairs on the COMPACTED list of such keys (128 consecutive list entries per
//                     unit, gathered K/V rows) against one chunk of the query range; every (list tile,
//                     query chunk) unit writes an fp32 partial dK/dV to the workspace.
//   dkv_kernel<band>: one workgroup per 128 consecutive keys against the queries j <= i < j+n.  Its
//                     epilogue adds, in fixed chunk order, the far partials of the keys that have
//                     them, then rounds once to bf16.  One workgroup owns each key row: no atomics,
//                     results are bit-reproducible.
// A workgroup is 8 waves = 4 key blocks of 32 keys x 2 roles.  The two waves of a key block split
// the four contractions so that each keeps only one operand matrix and one accumulator resident:
//   P-wave :  S = Q K^T   -> P = exp2(.)      -> dV^T += dO^T P     (holds K rows, dV^T)
//   dS-wave:  dP = dO V^T -> dS = P (dP - D)  -> dK^T += Q^T dS     (holds V rows, dK^T)
// P travels from the first to the second through a small LDS buffer (same lane, same register:
// both are 32x32 accumulator layouts), once per block of 32 queries, fenced by the block's
// workgroup barrier.  Query tiles (64 rows of Q and dO, plus LSE*log2e and D) stream through a ring
// of three LDS buffers filled by direct global->LDS loads issued two tiles ahead; with the ring the
// block barriers are the only barriers.  The tiles are stored unpadded with XOR-permuted 16-byte
// chunks so that both the row-major reads (first contraction) and the transposed reads (second
// contraction) are free of bank conflicts.  The four query heads of a GQA group are just four times
// as many query tiles.
#include "bwd_common.h"
#include "mfma_common.h"

namespace sepattn {

namespace {

__device__ inline int wave_min_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));
    return v;
}
__device__ inline int wave_max_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

template <int D, bool FAR>
__global__ __launch_bounds__(kDkvThreads, 1) void dkv_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const float *__restrict__ LSE2, const uint16_t *__restrict__ dO,
    const float *__restrict__ Dws, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ dK, uint16_t *__restrict__ dV,
    float *__restrict__ farK, float *__restrict__ farV) {
    constexpr int NW = 2 * kDkvWaves;        // waves per workgroup
    constexpr int CH = D / 8;                // 16-byte chunks per row
    constexpr int RPL = 64 / CH;             // rows covered by one wave-wide 1 KB load
    constexpr int LOADS = kBQ / (RPL * NW);  // wave-wide loads per wave per tensor per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    constexpr int TILE = kBQ * D;
    constexpr int NBUF = 3;
    static_assert(LOADS >= 1 && LOADS * RPL * NW == kBQ, "tile must divide among the waves");

    __shared__ __attribute__((aligned(1024))) uint16_t Qs[NBUF][TILE];
    __shared__ __attribute__((aligned(1024))) uint16_t dOs[NBUF][TILE];
    __shared__ __attribute__((aligned(256))) float lse_s[NBUF][kBQ];
    __shared__ __attribute__((aligned(256))) float d_s[NBUF][kBQ];
    __shared__ __attribute__((aligned(1024))) float Pex[kDkvWaves][2][4][64 * 4];  // [key block][qb][reg/4][lane*4]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave / kDkvWaves;  // 0: P-wave (S, dV), 1: dS-wave (dP, dK)
    const int kbw = wave % kDkvWaves;   // key block of the wave
    const int kj = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv;
    const int kv = blockIdx.y % p.Hkv, b = blockIdx.y / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const long kvrow0 = ((long)b * p.Hkv + kv) * (long)p.L;
    const float sl2 = p.scale * kLog2e_f;
    const FarGeom fg = far_geom(p);
    const FarList fl = far_list(p, prefix);
    const int a_row = pi_row(kj);
    const int my_pc = lane % CH, my_sub = lane / CH;
    // loads this wave issues per tile: the first two waves also fetch LSE*log2e and D
    const bool extra_load = wave < 2;

    const int n_units = FAR ? ((fl.NF + kBK - 1) / kBK) * fg.NCH : 1;
    bool first_unit = true;
    for (int unit = FAR ? (int)blockIdx.x : 0; unit < n_units; unit += FAR ? (int)gridDim.x : 1) {
        // ---- this wave's 32 keys and the query range of the unit
        int j, lo, hi, q_lo, q_hi, fidx = 0, chunk = 0;
        bool valid;
        if (FAR) {
            int ft = unit / fg.NCH;
            chunk = unit % fg.NCH;
            int pos_first = far_pos(fl, ft * kBK, idx, p.L);
            q_lo = max(chunk * fg.CQ, align_down32(pos_first + p.n));
            q_hi = min(p.L, (chunk + 1) * fg.CQ);
            if (q_lo >= q_hi) continue;
            fidx = ft * kBK + 32 * kbw + kj;
            valid = fidx < fl.NF;
            j = valid ? far_pos(fl, fidx, idx, p.L) : 0;
            lo = j + p.n;
            hi = q_hi - 1;
        } else {
            int j0 = blockIdx.x * kBK;
            j = j0 + 32 * kbw + kj;
            valid = j < p.L;
            q_lo = j0;
            q_hi = min(p.L, j0 + kBK + p.n - 1);
            lo = j;
            hi = min(j + p.n - 1, p.L - 1);
            if (!valid) j = 0;
        }
        if (!valid) {
            lo = kIntMax;
            hi = -1;
        }
        const int lo_min = wave_min_i(lo), lo_max = wave_max_i(lo);
        const int hi_min = wave_min_i(hi), hi_max = wave_max_i(hi);

        // resident B operand: K rows for the P-wave, V rows for the dS-wave
        bf16x8 breg[KSTEPS];
        {
            const uint16_t *brow = (role == 0 ? K : V) + (kvrow0 + j) * D;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
                breg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(brow + ks * 16 + 8 * hh));
        }
        f32x16 acc[DB];  // dV^T (P-wave) or dK^T (dS-wave) of the wave's keys
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

        const int n_qt = (q_hi - q_lo + kBQ - 1) / kBQ;
        const int n_tiles = G * n_qt;

        // tile tt -> LDS buffer tt%3: wave w fills rows (LOADS*w + u)*RPL .. +RPL-1 with one wave-wide
        // direct load per tensor; a lane owns physical chunk lane%CH of its row and fetches the
        // logical chunk the permutation maps there.  Rows past the sequence end are clamped (they are
        // masked by the [lo, hi] test: hi <= L-1).
        auto issue_tile = [&](int tt) {
            const int g = tt / n_qt, qt = tt - g * n_qt;
            const int buf = tt % NBUF;
            const long hrow0 = ((long)b * p.Hq + kv * G + g) * (long)p.L;
            const int qbase = q_lo + qt * kBQ;
            static_for<LOADS>([&](auto U) {
                constexpr int u = U;
                const int r = (LOADS * wave + u) * RPL + my_sub;
                const long row = hrow0 + min(qbase + r, p.L - 1);
                const int lc = swz_chunk<kSwzBoth, D>(my_pc, r);
                const int wave_off = (LOADS * wave + u) * RPL * D;
                load_to_lds_16(Q + row * D + lc * 8, &Qs[buf][wave_off]);
                load_to_lds_16(dO + row * D + lc * 8, &dOs[buf][wave_off]);
            });
            if (wave == 0) load_to_lds_4(LSE2 + hrow0 + min(qbase + lane, p.L - 1), &lse_s[buf][0]);
            if (wave == 1) load_to_lds_4(Dws + hrow0 + min(qbase + lane, p.L - 1), &d_s[buf][0]);
        };
        // wait until at most the loads of one tile (the newest) are still in flight; they complete
        // in the order they were issued
        auto wait_all_but_newest_tile = [&](bool newest_issued) {
            if (!newest_issued) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else if (extra_load) {
                if constexpr (LOADS == 1)
                    asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
                else
                    asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
            } else {
                if constexpr (LOADS == 1)
                    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                else
                    asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            }
        };
        static_assert(LOADS == 1 || LOADS == 2, "wait counts above are written for 1 or 2 loads per tensor");

        // the previous unit's last tile may still be read by other waves
        if (!first_unit) __syncthreads();
        first_unit = false;
        issue_tile(0);
        if (n_tiles > 1) issue_tile(1);
        wait_all_but_newest_tile(n_tiles > 1);
        __builtin_amdgcn_s_barrier();

        for (int tt = 0; tt < n_tiles; ++tt) {
            const int buf = tt % NBUF;
            // first contraction reads rows, second reads the other tensor transposed
            const uint16_t *T1 = role == 0 ? Qs[buf] : dOs[buf];
            const uint16_t *T2 = role == 0 ? dOs[buf] : Qs[buf];
            const float *rowval = role == 0 ? lse_s[buf] : d_s[buf];
            const int qb0 = q_lo + (tt % n_qt) * kBQ;

#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int r0 = qb0 + 32 * qb, r1 = r0 + 31;              // query rows of this block
                const bool active = !(r1 < lo_min || r0 > hi_max);       // any visible pair for this key block?
                const bool full = (r0 >= lo_max) && (r1 <= hi_min);
                float *pex = &Pex[kbw][qb][0][lane * 4];
                f32x16 x;
                if (active) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) x[i] = 0.f;
                    const int row = qb * 32 + a_row;
#pragma unroll
                    for (int ks = 0; ks < KSTEPS; ++ks)
                        x = mfma_bf16(lds_read_a_swz<kSwzBoth, D>(T1, row, 2 * ks + hh), breg[ks], x);
                    if (role == 0) {
                        // P = exp2(S*scale*log2e - LSE*log2e), zero where masked; hand it to the dS-wave
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int base = qb * 32 + 16 * half + 8 * hh;
                            const float4 l0 = *reinterpret_cast<const float4 *>(rowval + base);
                            const float4 l1 = *reinterpret_cast<const float4 *>(rowval + base + 4);
                            const float ls[8] = {l0.x, l0.y, l0.z, l0.w, l1.x, l1.y, l1.z, l1.w};
#pragma unroll
                            for (int k = 0; k < 8; ++k) {
                                const int i = 8 * half + k;
                                const int iqr = qb0 + base + k;
                                float pr = __builtin_amdgcn_exp2f(fmaf(x[i], sl2, -ls[k]));
                                if (!full) pr = (lo <= iqr && iqr <= hi) ? pr : 0.f;
                                x[i] = pr;
                            }
                        }
#pragma unroll
                        for (int g4 = 0; g4 < 4; ++g4) {
                            f32x4 v4 = {x[4 * g4], x[4 * g4 + 1], x[4 * g4 + 2], x[4 * g4 + 3]};
                            *reinterpret_cast<f32x4 *>(pex + g4 * 256) = v4;
                        }
                    }
                }
                // block barrier: P of this block is in LDS.  The second one of a tile also publishes
                // the next tile (every wave has waited for its own share of it).
                if (qb == 1) wait_all_but_newest_tile(tt + 2 < n_tiles);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                // after the first barrier of tile tt nobody reads tile tt-1 any more: refill its buffer
                if (qb == 0 && tt + 2 < n_tiles) issue_tile(tt + 2);
                if (active) {
                    if (role == 1) {
                        // dS = P (dP - D)
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int base = qb * 32 + 16 * half + 8 * hh;
                            const float4 d0 = *reinterpret_cast<const float4 *>(rowval + base);
                            const float4 d1 = *reinterpret_cast<const float4 *>(rowval + base + 4);
                            const float dd[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
                            const f32x4 p0 = *reinterpret_cast<const f32x4 *>(pex + (2 * half) * 256);
                            const f32x4 p1 = *reinterpret_cast<const f32x4 *>(pex + (2 * half + 1) * 256);
                            const float pp[8] = {p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
#pragma unroll
                            for (int k = 0; k < 8; ++k) x[8 * half + k] = pp[k] * (x[8 * half + k] - dd[k]);
                        }
                    }
#pragma unroll
                    for (int stp = 0; stp < 2; ++stp) {
                        const bf16x8 xb = pack_bf16x8(x, 8 * stp);
#pragma unroll
                        for (int db = 0; db < DB; ++db)
                            acc[db] = mfma_bf16(
                                lds_read_a_tr_swz<kSwzBoth, D>(T2, qb * 32 + stp * 16, db * 32, lane), xb, acc[db]);
                    }
                }
            }
        }

        // ---- epilogue: the P-wave owns dV, the dS-wave owns dK (times scale)
        const float oscale = role == 0 ? 1.f : p.scale;
        float *farX = role == 0 ? farV : farK;
        if (FAR) {
            if (valid) {
                long prow = ((((long)b * p.Hkv + kv) * fg.NCH + chunk) * fg.NFcap + fidx) * D;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        int col = db * 32 + 8 * i4 + 4 * hh;
                        float4 a = {acc[db][4 * i4] * oscale, acc[db][4 * i4 + 1] * oscale,
                                    acc[db][4 * i4 + 2] * oscale, acc[db][4 * i4 + 3] * oscale};
                        *reinterpret_cast<float4 *>(farX + prow + col) = a;
                    }
            }
        } else if (valid) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[db][i] *= oscale;
            // far partials of this key, if it is an initial token or a separator
            int f = -1;
            if (j < fl.a_eff)
                f = j;
            else if (prefix[j + 1] != prefix[j])
                f = fl.a_eff + prefix[j] - fl.sep_base;
            if (f >= 0 && f < fl.NF) {
                int pos_first = far_pos(fl, (f / kBK) * kBK, idx, p.L);
                int A = align_down32(pos_first + p.n);
                if (A < p.L) {
                    for (int c = A / fg.CQ; c < fg.NCH; ++c) {
                        long prow = ((((long)b * p.Hkv + kv) * fg.NCH + c) * fg.NFcap + f) * D;
#pragma unroll
                        for (int db = 0; db < DB; ++db)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {
                                int col = db * 32 + 8 * i4 + 4 * hh;
                                float4 a = *reinterpret_cast<const float4 *>(farX + prow + col);
                                acc[db][4 * i4] += a.x;
                                acc[db][4 * i4 + 1] += a.y;
                                acc[db][4 * i4 + 2] += a.z;
                                acc[db][4 * i4 + 3] += a.w;
                            }
                    }
                }
            }
            uint16_t *orow = (role == 0 ? dV : dK) + (kvrow0 + j) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    int col = db * 32 + 8 * i4 + 4 * hh;
                    *reinterpret_cast<uint2 *>(orow + col) =
                        pack_bf16x4(acc[db][4 * i4], acc[db][4 * i4 + 1], acc[db][4 * i4 + 2], acc[db][4 * i4 + 3]);
                }
        }
    }
}

template <int D>
int launch_dkv(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
               const int32_t *sep_prefix, uint16_t *dK, uint16_t *dV, float *farK, float *farV,
               hipStream_t st) {
    FarGeom fg = far_geom(p);
    dim3 kblock(kDkvThreads);
    int far_tiles_max = fg.NFcap / kBK;
    int far_grid = far_tiles_max * fg.NCH < kFarGrid ? far_tiles_max * fg.NCH : kFarGrid;
    {
        ProfScope prof(SEPATTN_K_BWD_DKV_FAR, st);
        hipLaunchKernelGGL((dkv_kernel<D, true>), dim3(far_grid, p.B * p.Hkv), kblock, 0, st, p, Q, K, V, lse2, dO,
                           Dws, sep_idx, sep_prefix, dK, dV, farK, farV);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_BWD_DKV_BAND, st);
    hipLaunchKernelGGL((dkv_kernel<D, false>), dim3((p.L + kBK - 1) / kBK, p.B * p.Hkv), kblock, 0, st, p, Q, K, V,
                       lse2, dO, Dws, sep_idx, sep_prefix, dK, dV, farK, farV);
    return launch_status();
}

}  // namespace

int launch_dkv_bf16(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                    const float *lse2, const uint16_t *dO, const float *Dws, const int32_t *sep_idx,
                    const int32_t *sep_prefix, uint16_t *dK, uint16_t *dV, float *farK, float *farV,
                    hipStream_t st) {
    if (p.d == 64) return launch_dkv<64>(p, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, dK, dV, farK, farV, st);
    return launch_dkv<128>(p, Q, K, V, lse2, dO, Dws, sep_idx, sep_prefix, dK, dV, farK, farV, st);
}

}  // namespace sepattn
