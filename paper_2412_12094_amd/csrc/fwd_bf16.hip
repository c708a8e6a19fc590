// SepAttention forward, bf16 MFMA (Eq. 1 with the mask of Eq. 2), flash-style with online softmax.
//
// A workgroup owns TP consecutive query positions of GP query heads that share one KV head
// (grouped-query attention: the heads are packed into the row dimension, so K/V tiles and the mask
// are shared).  Each wave owns 32 rows: one head, 32 positions.  The keys a tile can see are turned
// into ONE dense stream,
//     [ initial tokens j < min(a, bs) | separators in [min(a,bs), bs) | band keys bs .. i0+TP-1 ]
// with bs = max(0, i0-n+1) the first key of the first row's neighbour window (Sec. 3.1).  The first
// two parts are visible to every row of the tile (they are older than every window and are initial
// tokens / separators) and are gathered through the compacted separator index list; only band keys
// need the per-element test  j <= i and (i-j < n or j is an initial token or a separator).
//
// Pipeline per 64-key tile (LDS double-buffered, one barrier per tile):
//   meta(t+3): index / prefix loads  ->  rows(t+2): K,V row loads into registers
//   ->  store(t+1): registers to LDS stage (t+1)&1  ->  compute(t) from LDS stage t&1.
// S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_32x32x16_bf16 with V^T read by
// ds_read_b64_tr_b16; the LDS operand reads of a 32-key block are issued as one batch ahead of its
// MFMAs.  A wave skips 32-key blocks that lie entirely in its future and drops the mask test on
// blocks every one of its rows sees in full.  The running maximum is only raised when it grows by
// more than 2^8 (the accumulators stay exact: all terms carry the same stale maximum), which removes
// almost every rescale of the output accumulators.
#include "common.h"
#include "mfma_common.h"
#include "key_stream.h"

#ifdef SEPATTN_X_TIMING
__device__ unsigned long long g_dbg[8 * 8 * 2048];
extern "C" int sepattn_debug_read(unsigned long long *host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg), sizeof(unsigned long long) * n);
}
#define TICK(k)                                  \
    {                                            \
        unsigned long long now_ = clock64();     \
        tacc[k] += now_ - tlast;                 \
        tlast = now_;                            \
    }
#else
#define TICK(k)
#endif

namespace sepattn {

namespace {

constexpr float kRescaleThreshold = 8.f;  // log2 units

template <int D, int NW, int GP>
__global__ __launch_bounds__(NW * 64, 2) void fwd_bf16_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ O, float *__restrict__ LSE) {
    constexpr int NT = NW * 64;
    constexpr int TP = 32 * NW / GP;  // query positions per workgroup
    constexpr int KS = D + 8;         // LDS row strides in elements (bank spreading)
    constexpr int VS = D + 32;
    constexpr int CH = D / 8;             // 16-byte chunks per row
    constexpr int LOADS = kBN * CH / NT;  // rows per thread per tile (one chunk of each)
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    static_assert(kBN * CH % NT == 0 && LOADS >= 1, "tile must divide among the threads");

    __shared__ __attribute__((aligned(16))) uint16_t Ks[2][kBN * KS];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[2][kBN * VS];
    __shared__ __attribute__((aligned(16))) int lo_s[2][kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[2][kBN];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps branches scalar
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

    // ---- load pipeline state (per thread: LOADS rows, one 16-byte chunk of K and of V each)
    const int my_ch = tid % CH, my_r0 = tid / CH;  // row of load u is my_r0 + u * (NT / CH)
    int raw0[LOADS], raw1[LOADS];                  // meta stage: idx entry or prefix[j], prefix[j+1]
    u32x4 kpre[LOADS], vpre[LOADS];                // row stage
    int lo_pre[LOADS], hi_pre[LOADS];

    auto issue_meta = [&](int t) {
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            int k = t * kBN + my_r0 + u * (NT / CH);
            raw0[u] = 0;
            raw1[u] = 0;
            if (k >= st.n_init && k < st.n_dense) {
                raw0[u] = idx[min(st.sep_lo + k - st.n_init, p.cap - 1)];
            } else if (k >= st.n_dense && k < st.n_total) {
                int j = st.bs + (k - st.n_dense);
                raw0[u] = prefix[j];
                raw1[u] = prefix[j + 1];
            }
        });
    };
    auto issue_rows = [&](int t) {
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            int k = t * kBN + my_r0 + u * (NT / CH);
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
            lo_pre[u] = lo;
            hi_pre[u] = hi;
            kpre[u] = *reinterpret_cast<const u32x4 *>(Kh + (long)j * D + my_ch * 8);
            vpre[u] = *reinterpret_cast<const u32x4 *>(Vh + (long)j * D + my_ch * 8);
        });
    };
    auto store_tile = [&](int stage) {
        static_for<LOADS>([&](auto U) {
            constexpr int u = U;
            int r = my_r0 + u * (NT / CH);
            *reinterpret_cast<u32x4 *>(&Ks[stage][r * KS + my_ch * 8]) = kpre[u];
            *reinterpret_cast<u32x4 *>(&Vs[stage][r * VS + my_ch * 8]) = vpre[u];
            if (my_ch == 0) {
                lo_s[stage][r] = lo_pre[u];
                hi_s[stage][r] = hi_pre[u];
            }
        });
    };

    issue_meta(0);
    issue_rows(0);
    if (n_tiles > 1) issue_meta(1);
    store_tile(0);
    if (n_tiles > 1) issue_rows(1);
    if (n_tiles > 2) issue_meta(2);
    __syncthreads();

    const int a_row = pi_row(qi);
#ifdef SEPATTN_X_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tlast = clock64();
#endif
    for (int t = 0; t < n_tiles; ++t) {
        const int stage = t & 1;
        TICK(7)
        if (t + 1 < n_tiles) store_tile(stage ^ 1);
        if (t + 2 < n_tiles) issue_rows(t + 2);
        if (t + 3 < n_tiles) issue_meta(t + 3);

        TICK(0)
        const uint16_t *Kst = Ks[stage], *Vst = Vs[stage];
        // classify the two 32-key blocks for this wave: skip / all visible / test each pair
        int mode[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) mode[kb] = block_mode(st, t * kBN + kb * 32, pw, p.n);

        if (mode[0] != 0 || mode[1] != 0) {
            // ---- S^T = K Q^T: all operand reads of a block first, then its MFMAs
            f32x16 sacc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (mode[kb] == 0) continue;
                bf16x8 ka[KSTEPS];
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks)
                    ka[ks] = lds_read_a(Kst, kb * 32 + a_row, KS, ks * 16 + 8 * hh);
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) sacc[kb] = mfma_bf16(ka[ks], qreg[ks], sacc[kb]);
            }
            TICK(1)
            // ---- mask (only where needed) and block maximum of the raw scores
            float m_loc = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (mode[kb] == 0) continue;
                if (mode[kb] == 2) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        int base = kb * 32 + 16 * half + 8 * hh;
                        int4 lo0 = *reinterpret_cast<const int4 *>(&lo_s[stage][base]);
                        int4 lo1 = *reinterpret_cast<const int4 *>(&lo_s[stage][base + 4]);
                        int4 hi0 = *reinterpret_cast<const int4 *>(&hi_s[stage][base]);
                        int4 hi1 = *reinterpret_cast<const int4 *>(&hi_s[stage][base + 4]);
                        int los[8] = {lo0.x, lo0.y, lo0.z, lo0.w, lo1.x, lo1.y, lo1.z, lo1.w};
                        int his[8] = {hi0.x, hi0.y, hi0.z, hi0.w, hi1.x, hi1.y, hi1.z, hi1.w};
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            bool vis = (los[k] <= iq) && (iq <= his[k]);
                            sacc[kb][8 * half + k] = vis ? sacc[kb][8 * half + k] : -INFINITY;
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) m_loc = fmaxf(m_loc, sacc[kb][i]);
            }
            // ---- online softmax with a lazily raised maximum
            float m_new = fmaxf(m_run, pair_max(m_loc * sl2));
            bool grow = m_new > m_run + kRescaleThreshold;
            if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
                float alpha = grow ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
                m_run = grow ? m_new : m_run;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
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
            }
            l_run += psum;

            TICK(2)
            // ---- O^T += V^T P^T: the 16 transposed reads of a block first, then its 2*DB MFMAs
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                if (mode[kb] == 0) continue;
                bf16x8 vt[2][DB];
#pragma unroll
                for (int stp = 0; stp < 2; ++stp)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        vt[stp][db] = lds_read_a_tr(Vst, kb * 32 + stp * 16, VS, db * 32, lane);
#pragma unroll
                for (int stp = 0; stp < 2; ++stp) {
                    bf16x8 pb = pack_bf16x8(sacc[kb], 8 * stp);
#pragma unroll
                    for (int db = 0; db < DB; ++db) oacc[db] = mfma_bf16(vt[stp][db], pb, oacc[db]);
                }
            }
            TICK(3)
        }
        __syncthreads();  // stage^1 is complete for the next tile; everyone is done reading `stage`
        TICK(4)
    }
#ifdef SEPATTN_X_TIMING
    if (lane == 0 && blockIdx.x < 2048) {
        tacc[5] = n_tiles;
        for (int k = 0; k < 8; ++k) g_dbg[((long)blockIdx.x * 8 + wave) * 8 + k] = tacc[k];
    }
#endif

    // epilogue: normalise, store O (bf16) and LSE (natural log)
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

template <int D, int NW>
int launch_fwd(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const int32_t *sep_idx, const int32_t *sep_prefix, uint16_t *O, float *LSE,
               hipStream_t st) {
    int G = p.Hq / p.Hkv;
    int GP = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    int TP = 32 * NW / GP;
    dim3 grid(((p.L + TP - 1) / TP) * p.B * p.Hkv * (G / GP)), block(NW * 64);
    ProfScope prof(SEPATTN_K_FORWARD, st);
    if (GP == 4)
        hipLaunchKernelGGL((fwd_bf16_kernel<D, NW, 4>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    else if (GP == 2)
        hipLaunchKernelGGL((fwd_bf16_kernel<D, NW, 2>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    else
        hipLaunchKernelGGL((fwd_bf16_kernel<D, NW, 1>), grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, O, LSE);
    return launch_status();
}

}  // namespace

#ifndef SEPATTN_FWD_WAVES
#define SEPATTN_FWD_WAVES 8
#endif

size_t forward_bf16_workspace(const sepattn_params &) { return 0; }

int launch_forward_bf16(const sepattn_params &p, const void *Q, const void *K, const void *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, void *O, float *LSE,
                        void *, hipStream_t st) {
    auto q = static_cast<const uint16_t *>(Q), k = static_cast<const uint16_t *>(K),
         v = static_cast<const uint16_t *>(V);
    auto o = static_cast<uint16_t *>(O);
    if (p.d == 64) return launch_fwd<64, SEPATTN_FWD_WAVES>(p, q, k, v, sep_idx, sep_prefix, o, LSE, st);
    return launch_fwd<128, SEPATTN_FWD_WAVES>(p, q, k, v, sep_idx, sep_prefix, o, LSE, st);
}

}  // namespace sepattn
