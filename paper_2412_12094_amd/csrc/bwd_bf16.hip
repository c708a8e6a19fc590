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
#include "common.h"
#include "mfma_common.h"
#include "key_stream.h"

namespace sepattn {

namespace {

constexpr int kFarChunks = 16;  // at most this many query chunks for the far pass
constexpr int kFarChunkMin = 512;
constexpr int kDkvWaves = 4;
constexpr int kBK = 32 * kDkvWaves;  // keys per dK/dV workgroup
constexpr int kBQ = 64;              // queries per LDS tile in the dK/dV kernels
constexpr int kFarGrid = 1024;       // persistent workgroups per (batch, KV head) in the far pass

__device__ inline int align_down32(int x) { return x & ~31; }

struct FarGeom {
    int CQ, NCH, NFcap;
};
__host__ __device__ inline FarGeom far_geom(const sepattn_params &p) {
    FarGeom g;
    int cq = (p.L + kFarChunks - 1) / kFarChunks;
    cq = (cq + 31) / 32 * 32;
    g.CQ = cq < kFarChunkMin ? kFarChunkMin : cq;
    g.NCH = (p.L + g.CQ - 1) / g.CQ;
    g.NFcap = (p.a + p.cap + kBK - 1) / kBK * kBK;
    return g;
}

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
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ dQ, float *__restrict__ Dws) {
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

// ---------------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------------
__device__ inline int wave_min_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));
    return v;
}
__device__ inline int wave_max_i(int v) {
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

struct FarList {
    int a_eff, sep_base, NF;
};
__device__ inline FarList far_list(const sepattn_params &p, const int32_t *__restrict__ prefix) {
    FarList f;
    f.a_eff = p.a;  // already clamped to L by the host
    f.sep_base = prefix[f.a_eff];
    int cnt = min(prefix[p.L], p.cap);
    f.NF = f.a_eff + max(cnt - f.sep_base, 0);
    return f;
}
__device__ inline int far_pos(const FarList &fl, int f, const int32_t *__restrict__ idx, int L) {
    if (f < fl.a_eff) return f;
    return min(max(idx[fl.sep_base + f - fl.a_eff], 0), L - 1);
}

template <int D, bool FAR>
__global__ __launch_bounds__(kDkvWaves * 64) void dkv_kernel(
    sepattn_params p, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const float *__restrict__ LSE, const uint16_t *__restrict__ dO,
    const float *__restrict__ Dws, const int32_t *__restrict__ sep_idx,
    const int32_t *__restrict__ sep_prefix, uint16_t *__restrict__ dK, uint16_t *__restrict__ dV,
    float *__restrict__ farK, float *__restrict__ farV) {
    constexpr int NT = kDkvWaves * 64;
    constexpr int QS = D + 8;
    constexpr int CH = D / 8;
    constexpr int LOADS = kBQ * CH / NT;
    constexpr int KSTEPS = D / 16;
    constexpr int DB = D / 32;

    __shared__ __attribute__((aligned(16))) uint16_t Qs[kBQ * QS];
    __shared__ __attribute__((aligned(16))) uint16_t dOs[kBQ * QS];
    __shared__ __attribute__((aligned(16))) float lse_s[kBQ];
    __shared__ __attribute__((aligned(16))) float d_s[kBQ];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kj = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv;
    const int kv = blockIdx.y % p.Hkv, b = blockIdx.y / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    const long kvrow0 = ((long)b * p.Hkv + kv) * (long)p.L;
    const float sl2 = p.scale * kLog2e_f;
    const FarGeom fg = far_geom(p);
    const FarList fl = far_list(p, prefix);

    int n_units = FAR ? ((fl.NF + kBK - 1) / kBK) * fg.NCH : 1;
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
            fidx = ft * kBK + 32 * wave + kj;
            valid = fidx < fl.NF;
            j = valid ? far_pos(fl, fidx, idx, p.L) : 0;
            lo = j + p.n;
            hi = q_hi - 1;
        } else {
            int j0 = blockIdx.x * kBK;
            j = j0 + 32 * wave + kj;
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

        bf16x8 kreg[KSTEPS], vreg[KSTEPS];
        {
            const uint16_t *krow = K + (kvrow0 + j) * D, *vrow = V + (kvrow0 + j) * D;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                kreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(krow + ks * 16 + 8 * hh));
                vreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4 *>(vrow + ks * 16 + 8 * hh));
            }
        }
        f32x16 dk[DB], dv[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) dk[db][i] = dv[db][i] = 0.f;

        const int n_qt = (q_hi - q_lo + kBQ - 1) / kBQ;
        const int n_tiles = G * n_qt;

        u32x4 qpre[LOADS], dopre[LOADS];
        float lse_pre[LOADS], d_pre[LOADS];
        auto prefetch = [&](int tt) {
            int g = tt / n_qt, qt = tt % n_qt;
            long hrow0 = ((long)b * p.Hq + kv * G + g) * (long)p.L;
#pragma unroll
            for (int u = 0; u < LOADS; ++u) {
                int c = tid + u * NT;
                int r = c / CH, ch = c % CH;
                long row = hrow0 + min(q_lo + qt * kBQ + r, p.L - 1);
                qpre[u] = *reinterpret_cast<const u32x4 *>(Q + row * D + ch * 8);
                dopre[u] = *reinterpret_cast<const u32x4 *>(dO + row * D + ch * 8);
                if (ch == 0) {
                    lse_pre[u] = LSE[row] * kLog2e_f;
                    d_pre[u] = Dws[row];
                }
            }
        };
        prefetch(0);

        for (int tt = 0; tt < n_tiles; ++tt) {
            __syncthreads();
#pragma unroll
            for (int u = 0; u < LOADS; ++u) {
                int c = tid + u * NT;
                int r = c / CH, ch = c % CH;
                *reinterpret_cast<u32x4 *>(Qs + r * QS + ch * 8) = qpre[u];
                *reinterpret_cast<u32x4 *>(dOs + r * QS + ch * 8) = dopre[u];
                if (ch == 0) {
                    lse_s[r] = lse_pre[u];
                    d_s[r] = d_pre[u];
                }
            }
            __syncthreads();
            if (tt + 1 < n_tiles) prefetch(tt + 1);
            const int qb0 = q_lo + (tt % n_qt) * kBQ;

#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int r0 = qb0 + 32 * qb, r1 = r0 + 31;  // query rows of this block
                if (r1 < lo_min || r0 > hi_max) continue;     // no visible pair for this wave
                const bool full = (r0 >= lo_max) && (r1 <= hi_min);
                f32x16 sacc, pacc;
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = pacc[i] = 0.f;
                int row = qb * 32 + pi_row(kj);
#pragma unroll
                for (int ks = 0; ks < KSTEPS; ++ks) {
                    sacc = mfma_bf16(lds_read_a(Qs, row, QS, ks * 16 + 8 * hh), kreg[ks], sacc);
                    pacc = mfma_bf16(lds_read_a(dOs, row, QS, ks * 16 + 8 * hh), vreg[ks], pacc);
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    int base = qb * 32 + 16 * half + 8 * hh;
                    float4 l0 = *reinterpret_cast<const float4 *>(lse_s + base);
                    float4 l1 = *reinterpret_cast<const float4 *>(lse_s + base + 4);
                    float4 d0 = *reinterpret_cast<const float4 *>(d_s + base);
                    float4 d1 = *reinterpret_cast<const float4 *>(d_s + base + 4);
                    float ls[8] = {l0.x, l0.y, l0.z, l0.w, l1.x, l1.y, l1.z, l1.w};
                    float dd[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        int i = 8 * half + k;
                        int iqr = qb0 + base + k;
                        float pr = __builtin_amdgcn_exp2f(sacc[i] * sl2 - ls[k]);
                        if (!full) pr = (lo <= iqr && iqr <= hi) ? pr : 0.f;
                        sacc[i] = pr;
                        pacc[i] = pr * (pacc[i] - dd[k]);
                    }
                }
#pragma unroll
                for (int stp = 0; stp < 2; ++stp) {
                    bf16x8 pb = pack_bf16x8(sacc, 8 * stp);
                    bf16x8 dsb = pack_bf16x8(pacc, 8 * stp);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        bf16x8 dot = lds_read_a_tr(dOs, qb * 32 + stp * 16, QS, db * 32, lane);
                        dv[db] = mfma_bf16(dot, pb, dv[db]);
                        bf16x8 qt_ = lds_read_a_tr(Qs, qb * 32 + stp * 16, QS, db * 32, lane);
                        dk[db] = mfma_bf16(qt_, dsb, dk[db]);
                    }
                }
            }
        }

        // ---- epilogue
        if (FAR) {
            if (valid) {
                long prow = ((((long)b * p.Hkv + kv) * fg.NCH + chunk) * fg.NFcap + fidx) * D;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        int col = db * 32 + 8 * i4 + 4 * hh;
                        float4 a = {dk[db][4 * i4] * p.scale, dk[db][4 * i4 + 1] * p.scale,
                                    dk[db][4 * i4 + 2] * p.scale, dk[db][4 * i4 + 3] * p.scale};
                        float4 c4 = {dv[db][4 * i4], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]};
                        *reinterpret_cast<float4 *>(farK + prow + col) = a;
                        *reinterpret_cast<float4 *>(farV + prow + col) = c4;
                    }
            }
        } else if (valid) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) dk[db][i] *= p.scale;
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
                                float4 a = *reinterpret_cast<const float4 *>(farK + prow + col);
                                float4 c4 = *reinterpret_cast<const float4 *>(farV + prow + col);
                                dk[db][4 * i4] += a.x;
                                dk[db][4 * i4 + 1] += a.y;
                                dk[db][4 * i4 + 2] += a.z;
                                dk[db][4 * i4 + 3] += a.w;
                                dv[db][4 * i4] += c4.x;
                                dv[db][4 * i4 + 1] += c4.y;
                                dv[db][4 * i4 + 2] += c4.z;
                                dv[db][4 * i4 + 3] += c4.w;
                            }
                    }
                }
            }
            uint16_t *dkrow = dK + (kvrow0 + j) * D, *dvrow = dV + (kvrow0 + j) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    int col = db * 32 + 8 * i4 + 4 * hh;
                    *reinterpret_cast<uint2 *>(dkrow + col) =
                        pack_bf16x4(dk[db][4 * i4], dk[db][4 * i4 + 1], dk[db][4 * i4 + 2], dk[db][4 * i4 + 3]);
                    *reinterpret_cast<uint2 *>(dvrow + col) =
                        pack_bf16x4(dv[db][4 * i4], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]);
                }
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
    FarGeom fg = far_geom(p);
    size_t d_bytes = align_up((size_t)p.B * p.Hq * p.L * sizeof(float), 256);
    size_t far_bytes = align_up((size_t)p.B * p.Hkv * fg.NCH * fg.NFcap * D * sizeof(float), 256);
    float *Dws = static_cast<float *>(ws);
    float *farK = reinterpret_cast<float *>(static_cast<char *>(ws) + d_bytes);
    float *farV = reinterpret_cast<float *>(static_cast<char *>(ws) + d_bytes + far_bytes);

    int G = p.Hq / p.Hkv;
    int GP = (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    int TP = 32 * NW / GP;
    dim3 grid((p.L + TP - 1) / TP, p.B * p.Hkv * (G / GP)), block(NW * 64);
    {
    ProfScope prof(SEPATTN_K_BWD_DQ, st);
    if (GP == 4)
        hipLaunchKernelGGL((dq_kernel<D, NW, 4>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws);
    else if (GP == 2)
        hipLaunchKernelGGL((dq_kernel<D, NW, 2>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws);
    else
        hipLaunchKernelGGL((dq_kernel<D, NW, 1>), grid, block, 0, st, p, Q, K, V, O, LSE, dO, sep_idx, sep_prefix, dQ, Dws);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;

    dim3 kblock(kDkvWaves * 64);
    int far_tiles_max = fg.NFcap / kBK;
    int far_grid = far_tiles_max * fg.NCH < kFarGrid ? far_tiles_max * fg.NCH : kFarGrid;
    {
        ProfScope prof(SEPATTN_K_BWD_DKV_FAR, st);
        hipLaunchKernelGGL((dkv_kernel<D, true>), dim3(far_grid, p.B * p.Hkv), kblock, 0, st, p, Q, K, V, LSE, dO,
                           Dws, sep_idx, sep_prefix, dK, dV, farK, farV);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_BWD_DKV_BAND, st);
    hipLaunchKernelGGL((dkv_kernel<D, false>), dim3((p.L + kBK - 1) / kBK, p.B * p.Hkv), kblock, 0, st, p, Q, K, V,
                       LSE, dO, Dws, sep_idx, sep_prefix, dK, dV, farK, farV);
    return launch_status();
}

}  // namespace

size_t backward_bf16_workspace(const sepattn_params &p) {
    FarGeom fg = far_geom(p);
    size_t d_bytes = align_up((size_t)p.B * p.Hq * p.L * sizeof(float), 256);
    size_t far_bytes = align_up((size_t)p.B * p.Hkv * fg.NCH * fg.NFcap * p.d * sizeof(float), 256);
    return d_bytes + 2 * far_bytes;
}

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
