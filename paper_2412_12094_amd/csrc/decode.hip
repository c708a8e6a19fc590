// Single-query attention over the four-block KV cache (Sec. 3.2 "Generation", Sec. 3.3).
//
// Every valid cache entry is visible, so this is Eq. 1 with one query row per head and M = 1.  The
// work is a pure stream over K and V: HBM-bound (2 * entries * d * 2 bytes per (sequence, KV head),
// a few flops per byte).  Layout of the launch:
//   - a workgroup owns one (sequence, KV head) and one of `nsplit` contiguous slices of the valid
//     entries; all Hq/Hkv query heads of the group are processed together so K and V are read once;
//   - inside a wave, d/8 lanes cover one cache row with 16-byte loads (a wave load instruction
//     covers 64/(d/8) whole rows, i.e. whole cache lines), scores are reduced across those lanes
//     with DPP adds, and each lane group keeps its own online-softmax state;
//   - partial (max, sum, unnormalised output) triples are merged through LDS, written to the
//     workspace, and a second tiny kernel merges the `nsplit` slices.
// With ROPE (positions within the cache, Sec. 3.3 "Positional Encoding") the keys are stored without
// position encoding; a rotary score depends on the distance between query and key only, so instead
// of turning the key row the kernel turns the query by that distance: the lane that holds
// dimensions of the first half uses q_x cos - q_y sin, the one with the second half q_y cos + q_x sin
// (cos / sin of distance * frequency from the caller's table).
#include "common.h"
#include "decode_common.h"

namespace sepattn {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ inline float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

template <typename T>
__device__ inline void load8(const T *p, float (&v)[8]);
template <>
__device__ inline void load8<uint16_t>(const uint16_t *p, float (&v)[8]) {
    uint4 u = *reinterpret_cast<const uint4 *>(p);
    v[0] = bf16lo(u.x); v[1] = bf16hi(u.x); v[2] = bf16lo(u.y); v[3] = bf16hi(u.y);
    v[4] = bf16lo(u.z); v[5] = bf16hi(u.z); v[6] = bf16lo(u.w); v[7] = bf16hi(u.w);
}
template <>
__device__ inline void load8<float>(const float *p, float (&v)[8]) {
    float4 a = *reinterpret_cast<const float4 *>(p);
    float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// the same for cache rows, which a call reads exactly once: non-temporal hint
template <typename T>
__device__ inline void load8_stream(const T *p, float (&v)[8]);
template <>
__device__ inline void load8_stream<uint16_t>(const uint16_t *p, float (&v)[8]) {
    const uint4 u = nt_load(reinterpret_cast<const uint4 *>(p));
    v[0] = bf16lo(u.x); v[1] = bf16hi(u.x); v[2] = bf16lo(u.y); v[3] = bf16hi(u.y);
    v[4] = bf16lo(u.z); v[5] = bf16hi(u.z); v[6] = bf16lo(u.w); v[7] = bf16hi(u.w);
}
template <>
__device__ inline void load8_stream<float>(const float *p, float (&v)[8]) {
    const uint4 a = nt_load(reinterpret_cast<const uint4 *>(p)), b = nt_load(reinterpret_cast<const uint4 *>(p + 4));
    v[0] = __uint_as_float(a.x); v[1] = __uint_as_float(a.y); v[2] = __uint_as_float(a.z); v[3] = __uint_as_float(a.w);
    v[4] = __uint_as_float(b.x); v[5] = __uint_as_float(b.y); v[6] = __uint_as_float(b.z); v[7] = __uint_as_float(b.w);
}

// sum over the LPR (8 or 16) adjacent lanes that share a cache row; every lane gets the total
template <int LPR>
__device__ inline float row_sum(float v) {
    // DPP controls: quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E,
    // row_half_mirror = 0x141, row_mirror = 0x140
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
    if (LPR == 16)
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
    return v;
}

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;
constexpr int kRowsUnroll = 4;  // rows per lane group per iteration

// partial record: [0] running max (log2 domain), [1] running sum, [2..2+D) unnormalised output
template <int D>
struct Partial {
    static constexpr int kFloats = D + 2;
};

template <typename T, int D, int GT, bool ROPE>
__global__ __launch_bounds__(kDecodeThreads) void decode_split_kernel(
    sepkv_params p, int nsplit, const T *__restrict__ q, const T *__restrict__ Kc,
    const T *__restrict__ Vc, const int32_t *__restrict__ sizes, const float *__restrict__ rope, int n_pos,
    float *__restrict__ part) {
    constexpr int LPR = D / 8;         // lanes per cache row
    constexpr int RPW = kWave / LPR;   // rows per wave load
    constexpr int NSLOT = kDecodeWaves * RPW;
    constexpr int PF = Partial<D>::kFloats;
    __shared__ float red[GT * NSLOT * PF];

    const int G = p.Hq / p.Hkv;
    const int groups = G / GT;
    int split = blockIdx.x;
    int blk = blockIdx.y;
    int hg = blk % groups;
    int kv = (blk / groups) % p.Hkv;
    int sq = blk / (groups * p.Hkv);
    int h0 = kv * G + hg * GT;

    const CacheMap cm = cache_map(p, sizes + SEPKV_SIZES_COLS * sq);
    int nv = cm.n_init + cm.n_sep + cm.n_past + cm.n_loc;
    int per = (nv + nsplit - 1) / nsplit;
    per = (per + NSLOT - 1) / NSLOT * NSLOT;
    int e0 = split * per, e1 = min(nv, e0 + per);

    int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    int sub = lane / LPR, c = lane % LPR;
    int slot_id = wave * RPW + sub;

    const T *Kh = Kc + ((long)sq * p.Hkv + kv) * (long)p.c * D;
    const T *Vh = Vc + ((long)sq * p.Hkv + kv) * (long)p.c * D;

    float qv[GT][8];
    for (int g = 0; g < GT; ++g) {
        load8<T>(q + ((long)sq * p.Hq + h0 + g) * D + c * 8, qv[g]);
        for (int t = 0; t < 8; ++t) qv[g][t] *= p.scale * kLog2e;
    }
    // the other member of each rotary pair (dimension i <-> i + D/2), signed: -q_y for a lane of the
    // first half, +q_x for one of the second half
    float qo[ROPE ? GT : 1][8];
    const int f0 = (c % (LPR / 2)) * 8;  // first of this lane's eight frequencies
    if constexpr (ROPE) {
        const float sgn = (c >= LPR / 2) ? p.scale * kLog2e : -p.scale * kLog2e;
        for (int g = 0; g < GT; ++g) {
            load8<T>(q + ((long)sq * p.Hq + h0 + g) * D + ((c + LPR / 2) % LPR) * 8, qo[g]);
            for (int t = 0; t < 8; ++t) qo[g][t] *= sgn;
        }
    }
    float m[GT], l[GT], acc[GT][8];
    for (int g = 0; g < GT; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
        for (int t = 0; t < 8; ++t) acc[g][t] = 0.f;
    }

    for (int eb = e0 + slot_id; eb < e1; eb += NSLOT * kRowsUnroll) {
        float kr[kRowsUnroll][8], vr[kRowsUnroll][8];
        bool ok[kRowsUnroll];
#pragma unroll
        for (int u = 0; u < kRowsUnroll; ++u) {
            int e = eb + u * NSLOT;
            ok[u] = e < e1;
            int sl = decode_slot_of(cm, ok[u] ? e : e0);
            load8_stream<T>(Kh + (long)sl * D + c * 8, kr[u]);
            load8_stream<T>(Vh + (long)sl * D + c * 8, vr[u]);
        }
        float sc[GT][kRowsUnroll];
        if constexpr (ROPE) {
#pragma unroll
            for (int u = 0; u < kRowsUnroll; ++u) {
                // entry e sits at position e, the query at nv - 1
                const int dist = ok[u] ? (nv - 1) - (eb + u * NSLOT) : 0;
                const float *row = rope + (long)min(dist, n_pos - 1) * D + f0;
                float co[8], si[8];
                load8<float>(row, co);
                load8<float>(row + D / 2, si);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float s = 0.f;
#pragma unroll
                    for (int t = 0; t < 8; ++t) s = fmaf(fmaf(qv[g][t], co[t], qo[g][t] * si[t]), kr[u][t], s);
                    s = row_sum<LPR>(s);
                    sc[g][u] = ok[u] ? s : -INFINITY;
                }
            }
        } else {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) {
                    float s = 0.f;
#pragma unroll
                    for (int t = 0; t < 8; ++t) s = fmaf(qv[g][t], kr[u][t], s);
                    s = row_sum<LPR>(s);
                    sc[g][u] = ok[u] ? s : -INFINITY;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float mn = m[g];
#pragma unroll
            for (int u = 0; u < kRowsUnroll; ++u) mn = fmaxf(mn, sc[g][u]);
            // the first row of the iteration is always valid, so mn is finite here
            float alpha = exp2f(m[g] - mn);
            float ps[kRowsUnroll], psum = 0.f;
#pragma unroll
            for (int u = 0; u < kRowsUnroll; ++u) {
                ps[u] = exp2f(sc[g][u] - mn);
                psum += ps[u];
            }
            l[g] = l[g] * alpha + psum;
            m[g] = mn;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                float x = acc[g][t] * alpha;
#pragma unroll
                for (int u = 0; u < kRowsUnroll; ++u) x = fmaf(ps[u], vr[u][t], x);
                acc[g][t] = x;
            }
        }
    }

    // merge the NSLOT lane-group states of the workgroup
    for (int g = 0; g < GT; ++g) {
        float *r = red + (g * NSLOT + slot_id) * PF;
        if (c == 0) {
            r[0] = m[g];
            r[1] = l[g];
        }
        for (int t = 0; t < 8; ++t) r[2 + c * 8 + t] = acc[g][t];
    }
    __syncthreads();
    for (int item = threadIdx.x; item < GT * D; item += kDecodeThreads) {
        int g = item / D, col = item % D;
        const float *r = red + g * NSLOT * PF;
        float M = -INFINITY;
        for (int s2 = 0; s2 < NSLOT; ++s2) M = fmaxf(M, r[s2 * PF]);
        float lsum = 0.f, o = 0.f;
        for (int s2 = 0; s2 < NSLOT; ++s2) {
            float ms = r[s2 * PF];
            float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
            lsum = fmaf(wgt, r[s2 * PF + 1], lsum);
            o = fmaf(wgt, r[s2 * PF + 2 + col], o);
        }
        float *dst = part + (((long)sq * p.Hq + h0 + g) * nsplit + split) * PF;
        dst[2 + col] = o;
        if (col == 0) {
            dst[0] = M;
            dst[1] = lsum;
        }
    }
}

// merge the nsplit slices of one (sequence, head): one workgroup of D threads
template <typename T, int D>
__global__ void decode_merge_kernel(int nsplit, const float *__restrict__ part, T *__restrict__ out,
                                    float *__restrict__ lse) {
    constexpr int PF = Partial<D>::kFloats;
    long sh = blockIdx.x;
    int col = threadIdx.x;
    const float *r = part + sh * nsplit * PF;
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, r[s * PF]);
    float lsum = 0.f, o = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        float ms = r[s * PF];
        float wgt = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
        lsum = fmaf(wgt, r[s * PF + 1], lsum);
        o = fmaf(wgt, r[s * PF + 2 + col], o);
    }
    float val = (lsum > 0.f) ? o / lsum : 0.f;
    if constexpr (sizeof(T) == 2)
        out[sh * D + col] = decode_f32_to_bf16(val);
    else
        out[sh * D + col] = val;
    if (lse && col == 0) lse[sh] = (lsum > 0.f) ? (M + log2f(lsum)) * kLn2 : -INFINITY;
}

int pick_gt(int G) { return (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1; }

int pick_nsplit(const sepkv_params &p) {
    // aim at ~8 workgroups per compute unit, at least 256 rows per slice
    long pairs = (long)p.S * p.Hkv * ((p.Hq / p.Hkv) / pick_gt(p.Hq / p.Hkv));
    long want = (2048 + pairs - 1) / pairs;
    long max_by_rows = (p.c + 255) / 256;
    long ns = want < max_by_rows ? want : max_by_rows;
    return (int)(ns < 1 ? 1 : (ns > 64 ? 64 : ns));
}

template <typename T, int D, bool ROPE>
int launch_decode_t(const sepkv_params &p, const T *q, const T *Kc, const T *Vc, const int32_t *sizes,
                    const float *rope, int n_pos, T *out, float *lse, float *part, hipStream_t st) {
    int G = p.Hq / p.Hkv, GT = pick_gt(G), nsplit = pick_nsplit(p);
    dim3 grid(nsplit, p.S * p.Hkv * (G / GT)), block(kDecodeThreads);
    {
    ProfScope prof(SEPATTN_K_DECODE_SPLIT, st);
    if (GT == 4)
        hipLaunchKernelGGL((decode_split_kernel<T, D, 4, ROPE>), grid, block, 0, st, p, nsplit, q, Kc, Vc, sizes, rope, n_pos, part);
    else if (GT == 2)
        hipLaunchKernelGGL((decode_split_kernel<T, D, 2, ROPE>), grid, block, 0, st, p, nsplit, q, Kc, Vc, sizes, rope, n_pos, part);
    else
        hipLaunchKernelGGL((decode_split_kernel<T, D, 1, ROPE>), grid, block, 0, st, p, nsplit, q, Kc, Vc, sizes, rope, n_pos, part);
    }
    if (hipGetLastError() != hipSuccess) return SEPATTN_ERR_HIP;
    ProfScope prof(SEPATTN_K_DECODE_MERGE, st);
    hipLaunchKernelGGL((decode_merge_kernel<T, D>), dim3(p.S * p.Hq), dim3(D), 0, st, nsplit, part, out, lse);
    return launch_status();
}

}  // namespace

size_t decode_workspace(const sepkv_params &p) {
    int nsplit = decode_mfma_applicable(p) ? decode_mfma_nsplit(p) : pick_nsplit(p);
    return align_up((size_t)p.S * p.Hq * nsplit * (p.d + 2) * sizeof(float), 256);
}

template <typename T>
int launch_decode_valu(const sepkv_params &p, const void *q, const void *Kc, const void *Vc, const int32_t *sizes,
                       const float *rope, int n_pos, void *out, float *lse, float *part, hipStream_t st) {
    const T *q_ = (const T *)q, *K_ = (const T *)Kc, *V_ = (const T *)Vc;
    if (p.d == 64 && rope) return launch_decode_t<T, 64, true>(p, q_, K_, V_, sizes, rope, n_pos, (T *)out, lse, part, st);
    if (p.d == 64) return launch_decode_t<T, 64, false>(p, q_, K_, V_, sizes, rope, n_pos, (T *)out, lse, part, st);
    if (rope) return launch_decode_t<T, 128, true>(p, q_, K_, V_, sizes, rope, n_pos, (T *)out, lse, part, st);
    return launch_decode_t<T, 128, false>(p, q_, K_, V_, sizes, rope, n_pos, (T *)out, lse, part, st);
}

int launch_decode(const sepkv_params &p, const void *q, const void *Kc, const void *Vc,
                  const int32_t *sizes, const float *rope, int n_pos, void *out, float *lse, void *ws,
                  hipStream_t st) {
    float *part = static_cast<float *>(ws);
    if (decode_mfma_applicable(p)) {
        using T = uint16_t;
        const int nsplit = decode_mfma_nsplit(p);
        int rc = launch_decode_mfma(p, nsplit, (const T *)q, (const T *)Kc, (const T *)Vc, sizes, rope, n_pos, (T *)out, lse, part, st);
        if (rc != SEPATTN_OK || nsplit == 1) return rc;
        ProfScope prof(SEPATTN_K_DECODE_MERGE, st);
        if (p.d == 64)
            hipLaunchKernelGGL((decode_merge_kernel<T, 64>), dim3(p.S * p.Hq), dim3(64), 0, st, nsplit, part, (T *)out, lse);
        else
            hipLaunchKernelGGL((decode_merge_kernel<T, 128>), dim3(p.S * p.Hq), dim3(128), 0, st, nsplit, part, (T *)out, lse);
        return launch_status();
    }
    if (p.dtype == SEPATTN_BF16) return launch_decode_valu<uint16_t>(p, q, Kc, Vc, sizes, rope, n_pos, out, lse, part, st);
    return launch_decode_valu<float>(p, q, Kc, Vc, sizes, rope, n_pos, out, lse, part, st);
}

}  // namespace sepattn
