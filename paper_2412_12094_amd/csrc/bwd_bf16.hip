// SepAttention backward, bf16 MFMA: the analytic gradient of Eq. 1 under the mask of Eq. 2.
//
//   D_i = <dO_i, O_i>,  P_ij = exp(scale*<Q_i,K_j> - LSE_i),  dP_ij = <dO_i, V_j>,
//   dS_ij = P_ij (dP_ij - D_i),  dQ_i = scale sum_j dS_ij K_j,  dK_j = scale sum_i dS_ij Q_i,
//   dV_j = sum_i P_ij dO_i   (dK, dV summed over the query heads of the KV head).
//
// Three launches, no floating-point atomics (results are bit-reproducible):
//  1. dq_kernel: one workgroup per query tile, same dense key stream as the forward
//     [initial | separators older than the window | band].  Also writes D_i for the other two.
//  2. dkv_kernel<far>: the visible pairs split into band pairs (i-j < n) and far pairs (i-j >= n,
//     j an initial token or a separator).  Far pairs are handled on the COMPACTED list of such keys
//     (128 consecutive list entries per workgroup, gathered K/V rows) against a chunk of the query
//     range; every (list tile, query chunk) unit writes an fp32 partial dK/dV to the workspace.
//  3. dkv_kernel<band>: one workgroup per 128 consecutive keys against the queries j <= i < j+n.
//     Its epilogue adds, in fixed chunk order, the far partials of the keys that have them, then
//     rounds once to bf16.  One workgroup owns each key row: no atomics needed.
// In the dK/dV kernels the wave's 32 keys are the B operands (kept in registers for the whole
// unit) and query tiles (Q, dO, LSE, D) stream through LDS; the four query heads of a GQA group are
// just four times as many query tiles.
#include "bwd_common.h"
#include "mfma_common.h"
#include "key_stream.h"

namespace sepattn {

namespace {

__device__ inline float bf16_dot8(u32x4 a, u32x4 b) {
    float s = 0.f;
    const uint32_t *x = reinterpret_cast<const uint32_t *>(&a);
    const uint32_t *y = reinterpret_cast<const uint32_t *>(&b);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        s = fmaf(__uint_as_float(x[k] << 16), __uint_as_float(y[k] << 16), s);
        s = fmaf(__uint_as_float(x[k] & 0xFFFF0000u), __uint_as_float(y[k] & 0xFFFF0000u), s);
    }
    return s;
}

// ---------------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------------
template <int D, int NW, int GP>
__global__ __launch_bounds__(NW * 64) void dq_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const uint16_t *__restrict__ O, const float *__restrict__ LSE,
    const uint16_t *__restrict__ dO, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ dQ, float *__restrict__ Dws,
    float *__restrict__ Lws) {
    constexpr int NT = NW * 64;
    constexpr int TP = 32 * NW / GP;
    constexpr int KS = D + 8;
    constexpr int CH = D / 8;
    constexpr int LOADS = kBN * CH / NT;
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;

    __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * KS];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[kBN * KS];
    __shared__ __attribute__((aligned(16))) int lo_s[kBN];
    __shared__ __attribute__((aligned(16))) int hi_s[kBN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv, groups = G / GP;
    const int tile = gridDim.x - 1 - blockIdx.x;
    const int i0 = tile * TP;
    int y = blockIdx.y;
    const int hg = y % groups;
    const int kv = (y / groups) % p.Hkv;
    const int b = y / (groups * p.Hkv);
    const int head = kv * G + hg * GP + (wave % GP);
    const int pw = i0 + 32 * (wave / GP);
    const int iq = pw + qi;

    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const uint16_t *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const uint16_t *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const Stream st = make_stream(p, prefix, i0, TP);
    const int n_tiles = (st.n_total + kBN - 1) / kBN;

    const long qrow_id = ((long)b * p.Hq + head) * p.L + min(iq, p.L - 1);
    bf16x8 qreg[KSTEPS], doreg[KSTEPS];
    float Di;
    {
        const uint16_t *qrow = Q + qrow_id * D, *dorow = dO + qrow_id * D, *orow = O + qrow_id * D;
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            u32x4 dq4 = *reinterpret_cast<const u32x4 *>(dorow + ks * 16 + 8 * hh);
            u32x4 o4 = *reinterpret_cast<const u32x4 *>(orow + ks * 16 + 8 * hh);
            qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(qrow + ks * 16 + 8 * hh));
            doreg[ks] = as_bf16x8(dq4);
            part += bf16_dot8(dq4, o4);
        }
        Di = pair_sum(part);
        if (hh == 0 && iq < p.L) Dws[qrow_id] = Di;
    }
    const float sl2 = p.scale * kLog2e_f;
    const float lse2 = LSE[qrow_id] * kLog2e_f;
    if (hh == 0 && iq < p.L) Lws[qrow_id] = lse2;  // the dK/dV kernels work in the log2 domain too

    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

    u32x4 kpre[LOADS], vpre[LOADS];
    int lo_pre[LOADS], hi_pre[LOADS];
    auto prefetch = [&](int t) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            int c = tid + u * NT;
            int r = c / CH, ch = c % CH;
            int j = stream_key(st, t * kBN + r, p, idx, prefix, lo_pre[u], hi_pre[u]);
            kpre[u] = *reinterpret_cast<const u32x4 *>(Kh + (long)j * D + ch * 8);
            vpre[u] = *reinterpret_cast<const u32x4 *>(Vh + (long)j * D + ch * 8);
        }
    };
    prefetch(0);

    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            int c = tid + u * NT;
            int r = c / CH, ch = c % CH;
            *reinterpret_cast<u32x4 *>(Ks + r * KS + ch * 8) = kpre[u];
            *reinterpret_cast<u32x4 *>(Vs + r * KS + ch * 8) = vpre[u];
            if (ch == 0) {
                lo_s[r] = lo_pre[u];
                hi_s[r] = hi_pre[u];
            }
        }
        __syncthreads();
        if (t + 1 < n_tiles) prefetch(t + 1);

#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            int mode = block_mode(st, t * kBN + kb * 32, pw, p.n);
            if (mode == 0) continue;
            f32x16 sacc, pacc;
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[i] = pacc[i] = 0.f;
            int row = kb * 32 + pi_row(qi);
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                sacc = mfma_bf16(lds_read_a(Ks, row, KS, ks * 16 + 8 * hh), qreg[ks], sacc);
                pacc = mfma_bf16(lds_read_a(Vs, row, KS, ks * 16 + 8 * hh), doreg[ks], pacc);
            }
            if (mode == 1) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float pr = __builtin_amdgcn_exp2f(sacc[i] * sl2 - lse2);
                    sacc[i] = pr * (pacc[i] - Di);
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
                        bool vis = (los[k] <= iq) & (iq <= his[k]);
                        float pr = __builtin_amdgcn_exp2f(sacc[i] * sl2 - lse2);
                        sacc[i] = vis ? pr * (pacc[i] - Di) : 0.f;
                    }
                }
            }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int stp = 0; stp < 2; ++stp) {
                bf16x8 dsb = pack_bf16x8(sacc, 8 * stp);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    bf16x8 kt = lds_read_a_tr(Ks, kb * 32 + stp * 16, KS, db * 32, lane);
                    acc[db] = mfma_bf16(kt, dsb, acc[db]);
                }
            }
        }
    }

    if (iq < p.L) {
        uint16_t *dst = dQ + qrow_id * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                uint2 v = pack_bf16x4(acc[db][4 * i4] * p.scale, acc[db][4 * i4 + 1] * p.scale,
                                      acc[db][4 * i4 + 2] * p.scale, acc[db][4 * i4 + 3] * p.scale);
                *reinterpret_cast<uint2 *>(dst + db * 32 + 8 * i4 + 4 * hh) = v;
            }
    }
}

#ifndef SEPATTN_DQ_WAVES
#define SEPATTN_DQ_WAVES 8
#endif

template <int D>
int launch_bwd(const sepattn_params &p, const uint16_t *Q, const uint16_t *K, const uint16_t *V,
               const uint16_t *O, const float *LSE, const uint16_t *dO, const int32_t *sep_idx,
               const int32_t *sep_prefix, uint16_t *dQ, uint16_t *dK, uint16_t *dV, void *ws,
               hipStream_t st) {
    constexpr int NW = SEPATTN_DQ_WAVES;
    const BwdWorkspace w = bwd_workspace(p);
    char *base = static_cast<char *>(ws);
    float *Dws = reinterpret_cast<float *>(base);
    float *Lws = reinterpret_cast<float *>(base + w.d_bytes);
    float *farK = reinterpret_cast<float *>(base + 2 * w.d_bytes);
    float *farV = reinterpret_cast<float *>(base + 2 * w.d_bytes + w.far_bytes);

    int G = p.Hq / p.Hkv;
    int GP = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    int TP = 32 * NW / GP;
    dim3 grid((p.L + TP - 1) / TP, p.B * p.Hkv * (G / GP)), block(NW * 64);
    {
    ProfScope prof(SEPATTN_K_BWD_DQ, st);
    if (GP == 4)
        hipLaunchKernelGGL((dq_kernel<D, NW, 4>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws, Lws);
    else if (GP == 2)
        hipLaunchKernelGGL((dq_kernel<D, NW, 2>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws, Lws);
    else
        hipLaunchKernelGGL((dq_kernel<D, NW, 1>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws, Lws);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    return launch_dkv_bf16(p, Q, K, V, Lws, dO, Dws, sep_idx, sep_prefix, dK, dV, farK, farV, st);
}

}  // namespace

size_t backward_bf16_workspace(const sepattn_params &p) { return bwd_workspace(p).total; }

int launch_backward_bf16(const sepattn_params &p, const void *Q, const void *K, const void *V,
                         const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                         const int32_t *, const int32_t *sep_prefix, void *dQ, void *dK, void *dV,
                         void *ws, hipStream_t st) {
    auto u = [](const void *x) { return static_cast<const uint16_t *>(x); };
    auto w = [](void *x) { return static_cast<uint16_t *>(x); };
    if (p.d == 64)
        return launch_bwd<64>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, w(dQ), w(dK), w(dV), ws, st);
    return launch_bwd<128>(p, u(Q), u(K), u(V), u(O), LSE, u(dO), sep_idx, sep_prefix, w(dQ), w(dK), w(dV), ws, st);
}

}  // namespace sepattn
