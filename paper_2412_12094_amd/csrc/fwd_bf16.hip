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
// The stream is cut into tiles of 64 keys; K and V rows are staged row-major in LDS (software
// prefetch of the next tile into registers); S^T = K Q^T and O^T += V^T P^T run on
// v_mfma_f32_32x32x16_bf16 with V^T read by ds_read_b64_tr_b16.  A wave skips 32-key blocks that lie
// entirely in its future and drops the mask test on blocks every one of its rows sees in full.
#include "common.h"
#include "mfma_common.h"
#include "key_stream.h"

namespace sepattn {

namespace {

template <int D, int NW, int GP>
__global__ __launch_bounds__(NW * 64) void fwd_bf16_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ O, float *__restrict__ LSE) {
    constexpr int NT = NW * 64;
    constexpr int TP = 32 * NW / GP;  // query positions per workgroup
    constexpr int KS = D + 8;         // LDS row strides (elements): see bank notes in the design doc
    constexpr int VS = D + 32;
    constexpr int CH = D / 8;                 // 16-byte chunks per row
    constexpr int LOADS = kBN * CH / NT;      // chunks per thread per tensor per tile
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;
    static_assert(kBN * CH % NT == 0, "tile must divide among the threads");

    __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * KS];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[kBN * VS];
    __shared__ __attribute__((aligned(16))) int lo_s[kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[kBN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv, groups = G / GP;
    const int tile = gridDim.x - 1 - blockIdx.x;  // late tiles carry more separators: start them first
    const int i0 = tile * TP;
    int y = blockIdx.y;
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
            qreg[ks] = as_bf16x8(*reinterpret_cast<const uint4 *>(qrow + ks * 16 + 8 * hh));
    }
    const float sl2 = p.scale * kLog2e_f;

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // software prefetch registers
    uint4 kpre[LOADS], vpre[LOADS];
    int lo_pre[LOADS], hi_pre[LOADS];
    auto prefetch = [&](int t) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            int c = tid + u * NT;
            int r = c / CH, ch = c % CH;
            int j = stream_key(st, t * kBN + r, p, idx, prefix, lo_pre[u], hi_pre[u]);
            kpre[u] = *reinterpret_cast<const uint4 *>(Kh + (long)j * D + ch * 8);
            vpre[u] = *reinterpret_cast<const uint4 *>(Vh + (long)j * D + ch * 8);
        }
    };
    prefetch(0);

    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();  // everyone is done reading the previous tile
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            int c = tid + u * NT;
            int r = c / CH, ch = c % CH;
            *reinterpret_cast<uint4 *>(Ks + r * KS + ch * 8) = kpre[u];
            *reinterpret_cast<uint4 *>(Vs + r * VS + ch * 8) = vpre[u];
            if (ch == 0) {
                lo_s[r] = lo_pre[u];
                hi_s[r] = hi_pre[u];
            }
        }
        __syncthreads();
        if (t + 1 < n_tiles) prefetch(t + 1);

        // classify the two 32-key blocks for this wave: skip / all visible / test each pair
        int mode[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) mode[kb] = block_mode(st, t * kBN + kb * 32, pw, p.n);
        if (mode[0] == 0 && mode[1] == 0) continue;

        // S^T = K Q^T for the active blocks
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
            if (mode[kb] != 0) {
                int row = kb * 32 + pi_row(qi);
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks)
                    sacc[kb] = mfma_bf16(lds_read_a(Ks, row, KS, ks * 16 + 8 * hh), qreg[ks], sacc[kb]);
            }
        }
        // scale into the log2 domain, mask, running maximum
        float m_loc = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (mode[kb] == 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[kb][i] = -INFINITY;
            } else if (mode[kb] == 1) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    sacc[kb][i] *= sl2;
                    m_loc = fmaxf(m_loc, sacc[kb][i]);
                }
            } else {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    int base = kb * 32 + 16 * half + 8 * hh;
                    int4 lo0 = *reinterpret_cast<const int4 *>(lo_s + base);
                    int4 lo1 = *reinterpret_cast<const int4 *>(lo_s + base + 4);
                    int4 hi0 = *reinterpret_cast<const int4 *>(hi_s + base);
                    int4 hi1 = *reinterpret_cast<const int4 *>(hi_s + base + 4);
                    int los[8] = {lo0.x, lo0.y, lo0.z, lo0.w, lo1.x, lo1.y, lo1.z, lo1.w};
                    int his[8] = {hi0.x, hi0.y, hi0.z, hi0.w, hi1.x, hi1.y, hi1.z, hi1.w};
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        int i = 8 * half + k;
                        bool vis = (los[k] <= iq) && (iq <= his[k]);
                        float s = vis ? sacc[kb][i] * sl2 : -INFINITY;
                        sacc[kb][i] = s;
                        m_loc = fmaxf(m_loc, s);
                    }
                }
            }
        }
        float m_new = fmaxf(m_run, pair_max(m_loc));
        float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float pr = __builtin_amdgcn_exp2f(sacc[kb][i] - m_safe);
                sacc[kb][i] = pr;
                psum += pr;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;

        // O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            if (mode[kb] == 0) continue;
#pragma unroll
            for (int stp = 0; stp < 2; ++stp) {
                bf16x8 pb = pack_bf16x8(sacc[kb], 8 * stp);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    bf16x8 vt = lds_read_a_tr(Vs, kb * 32 + stp * 16, VS, db * 32, lane);
                    oacc[db] = mfma_bf16(vt, pb, oacc[db]);
                }
            }
        }
    }

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
    dim3 grid((p.L + TP - 1) / TP, p.B * p.Hkv * (G / GP)), block(NW * 64);
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
