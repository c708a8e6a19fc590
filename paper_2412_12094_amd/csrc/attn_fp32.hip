// fp32 debug path of SepAttention forward and backward (Eq. 1 with the mask of Eq. 2).
//
// Slow and simple on purpose: one wavefront per query row (forward, dQ) or per key row (dK/dV),
// plain fp32 FMA arithmetic, no matrix cores.  It exists to validate the decomposition of a row's
// visible keys into  [initial tokens | separators older than the window | window]  (Sec. 3.1)
// against the oracle at tight tolerance, independently of the bf16 MFMA kernels.
//
// Row i sees: j < min(a, ws) (initial), separators in [min(a, ws), ws) (taken from the compacted
// index list), and the window ws <= j <= i with ws = max(0, i-n+1).  The three ranges are disjoint,
// so every visible pair is visited exactly once and no mask test is needed.
// Key j is seen by the contiguous query range [j, j+n) and, if it is an initial token or a
// separator, by every later query as well.
// Packed documents (doc_start / doc_end given, per position; the documents' initial tokens are
// marked in the bitmap and a = 0): the three ranges of a row start at its document's first position
// instead of 0, and a key's query range ends with its document.
#include "common.h"

namespace sepattn {

namespace {

template <int D>
__device__ inline float dot_row(const float *__restrict__ x, const float *__restrict__ y) {
    float s = 0.f;
#pragma unroll 8
    for (int k = 0; k < D; k += 4) {
        float4 a = *reinterpret_cast<const float4 *>(x + k);
        float4 b = *reinterpret_cast<const float4 *>(y + k);
        s = fmaf(a.x, b.x, s);
        s = fmaf(a.y, b.y, s);
        s = fmaf(a.z, b.z, s);
        s = fmaf(a.w, b.w, s);
    }
    return s;
}

__device__ inline float wave_max(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ inline float wave_sum(float v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

struct RowKeys {
    int n_init, n_sep, sep_lo, ws, total, ds;
};

// ds: first position of the row's document (0 without packing)
__device__ inline RowKeys row_keys(int i, int a, int n, const int32_t *__restrict__ prefix, int ds) {
    RowKeys r;
    r.ds = ds;
    r.ws = max(ds, i - n + 1);
    r.n_init = min(a, r.ws - ds);
    r.sep_lo = prefix[ds + r.n_init];
    r.n_sep = prefix[r.ws] - r.sep_lo;
    r.total = r.n_init + r.n_sep + (i - r.ws + 1);
    return r;
}

// cap and L bound the index read and the position it yields, so that a caller breaking
// sep_count <= cap (stale list tail) gets wrong numbers rather than a fault
__device__ inline int key_at(const RowKeys &r, int t, const int32_t *__restrict__ sep_idx, int cap, int L) {
    if (t < r.n_init) return r.ds + t;
    if (t < r.n_init + r.n_sep)
        return min(max(sep_idx[min(r.sep_lo + t - r.n_init, cap - 1)], 0), L - 1);
    return r.ws + (t - r.n_init - r.n_sep);
}

// ---- forward: one wave per (b, h, i) ---------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void fwd_fp32_kernel(sepattn_params p, const float *__restrict__ Q,
                                                       const float *__restrict__ K,
                                                       const float *__restrict__ V,
                                                       const int32_t *__restrict__ sep_idx,
                                                       const int32_t *__restrict__ sep_prefix,
                                                       const int32_t *__restrict__ doc_start,
                                                       float *__restrict__ O, float *__restrict__ LSE, HeadWin hw) {
    constexpr int R = D / kWave;  // output values per lane
    int lane = threadIdx.x % kWave;
    long row = (long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    long n_rows = (long)p.B * p.Hq * p.L;
    if (row >= n_rows) return;
    int i = (int)(row % p.L);
    int h = (int)((row / p.L) % p.Hq);
    int b = (int)(row / ((long)p.L * p.Hq));
    int kv = h / (p.Hq / p.Hkv);
    const float *q = Q + row * D;
    const float *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const float *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    // (the clamp keeps inconsistent bounds from faulting)
    RowKeys rk = row_keys(i, p.a, p.n - head_delta(hw, h), prefix, doc_start ? min(max(doc_start[(long)b * p.L + i], 0), i) : 0);

    float m = -INFINITY, l = 0.f;
    float acc[R];
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    for (int t0 = 0; t0 < rk.total; t0 += kWave) {
        int t = t0 + lane;
        int j = (t < rk.total) ? key_at(rk, t, idx, p.cap, p.L) : 0;
        float s = (t < rk.total) ? p.scale * dot_row<D>(q, Kh + (long)j * D) : -INFINITY;
        float m_new = fmaxf(m, wave_max(s));  // finite: the chunk holds at least one key
        float alpha = expf(m - m_new);
        float pr = expf(s - m_new);
        l = l * alpha + wave_sum(pr);
        for (int r = 0; r < R; ++r) acc[r] *= alpha;
        int cnt = min(kWave, rk.total - t0);
        for (int k = 0; k < cnt; ++k) {
            float pk = __shfl(pr, k);
            int jk = __shfl(j, k);
            for (int r = 0; r < R; ++r) acc[r] = fmaf(pk, Vh[(long)jk * D + lane + r * kWave], acc[r]);
        }
        m = m_new;
    }
    for (int r = 0; r < R; ++r) O[row * D + lane + r * kWave] = acc[r] / l;
    if (lane == 0) LSE[row] = m + logf(l);
}

// ---- backward pre-pass: D_i = <dO_i, O_i>, one wave per row -----------------------------------
template <int D>
__global__ __launch_bounds__(256) void rowdot_fp32_kernel(long n_rows, const float *__restrict__ dO,
                                                          const float *__restrict__ O,
                                                          float *__restrict__ Dout) {
    int lane = threadIdx.x % kWave;
    long row = (long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= n_rows) return;
    float s = 0.f;
    for (int k = lane; k < D; k += kWave) s = fmaf(dO[row * D + k], O[row * D + k], s);
    s = wave_sum(s);
    if (lane == 0) Dout[row] = s;
}

// ---- dQ: one wave per (b, h, i) -----------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void dq_fp32_kernel(sepattn_params p, const float *__restrict__ Q,
                                                      const float *__restrict__ K,
                                                      const float *__restrict__ V,
                                                      const float *__restrict__ LSE,
                                                      const float *__restrict__ dO,
                                                      const float *__restrict__ Drow,
                                                      const int32_t *__restrict__ sep_idx,
                                                      const int32_t *__restrict__ sep_prefix,
                                                      const int32_t *__restrict__ doc_start,
                                                      float *__restrict__ dQ, HeadWin hw) {
    constexpr int R = D / kWave;
    int lane = threadIdx.x % kWave;
    long row = (long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    long n_rows = (long)p.B * p.Hq * p.L;
    if (row >= n_rows) return;
    int i = (int)(row % p.L);
    int h = (int)((row / p.L) % p.Hq);
    int b = (int)(row / ((long)p.L * p.Hq));
    int kv = h / (p.Hq / p.Hkv);
    const float *q = Q + row * D;
    const float *go = dO + row * D;
    const float *Kh = K + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const float *Vh = V + ((long)b * p.Hkv + kv) * (long)p.L * D;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    const int32_t *idx = sep_idx + (long)b * p.cap;
    // (the clamp keeps inconsistent bounds from faulting)
    RowKeys rk = row_keys(i, p.a, p.n - head_delta(hw, h), prefix, doc_start ? min(max(doc_start[(long)b * p.L + i], 0), i) : 0);
    float lse = LSE[row], Di = Drow[row];
    float acc[R];
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    for (int t0 = 0; t0 < rk.total; t0 += kWave) {
        int t = t0 + lane;
        int j = 0;
        float ds = 0.f;
        if (t < rk.total) {
            j = key_at(rk, t, idx, p.cap, p.L);
            float s = p.scale * dot_row<D>(q, Kh + (long)j * D);
            float pr = expf(s - lse);
            float dp = dot_row<D>(go, Vh + (long)j * D);
            ds = pr * (dp - Di);
        }
        int cnt = min(kWave, rk.total - t0);
        for (int k = 0; k < cnt; ++k) {
            float dsk = __shfl(ds, k);
            int jk = __shfl(j, k);
            for (int r = 0; r < R; ++r) acc[r] = fmaf(dsk, Kh[(long)jk * D + lane + r * kWave], acc[r]);
        }
    }
    for (int r = 0; r < R; ++r) dQ[row * D + lane + r * kWave] = p.scale * acc[r];
}

// ---- dK, dV: one wave per (b, kv, j), loops over the query heads of the group and the queries
// that see key j ------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void dkv_fp32_kernel(sepattn_params p, const float *__restrict__ Q,
                                                       const float *__restrict__ K,
                                                       const float *__restrict__ V,
                                                       const float *__restrict__ LSE,
                                                       const float *__restrict__ dO,
                                                       const float *__restrict__ Drow,
                                                       const int32_t *__restrict__ sep_prefix,
                                                       const int32_t *__restrict__ doc_end,
                                                       float *__restrict__ dK, float *__restrict__ dV, HeadWin hw) {
    constexpr int R = D / kWave;
    int lane = threadIdx.x % kWave;
    long row = (long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    long n_rows = (long)p.B * p.Hkv * p.L;
    if (row >= n_rows) return;
    int j = (int)(row % p.L);
    int kv = (int)((row / p.L) % p.Hkv);
    int b = (int)(row / ((long)p.L * p.Hkv));
    int G = p.Hq / p.Hkv;
    const int32_t *prefix = sep_prefix + (long)b * (p.L + 1);
    bool always = (j < p.a) || (prefix[j + 1] != prefix[j]);
    const float *kj = K + row * D;
    const float *vj = V + row * D;
    float accK[R], accV[R];
    for (int r = 0; r < R; ++r) accK[r] = accV[r] = 0.f;
    for (int g = 0; g < G; ++g) {
        int h = kv * G + g;
        // the queries that see key j: up to the end of the sequence (document), or of head h's window
        long i_end_l = always ? (long)p.L : min((long)p.L, (long)j + p.n - head_delta(hw, h));
        if (doc_end) i_end_l = min(i_end_l, (long)doc_end[(long)b * p.L + j]);
        int i_end = (int)i_end_l;
        long hrow = ((long)b * p.Hq + h) * p.L;
        const float *Qh = Q + hrow * D;
        const float *dOh = dO + hrow * D;
        for (int i0 = j; i0 < i_end; i0 += kWave) {
            int i = i0 + lane;
            float pr = 0.f, ds = 0.f;
            if (i < i_end) {
                float s = p.scale * dot_row<D>(Qh + (long)i * D, kj);
                pr = expf(s - LSE[hrow + i]);
                float dp = dot_row<D>(dOh + (long)i * D, vj);
                ds = pr * (dp - Drow[hrow + i]);
            }
            int cnt = min(kWave, i_end - i0);
            for (int k = 0; k < cnt; ++k) {
                float pk = __shfl(pr, k);
                float dsk = __shfl(ds, k);
                long ik = i0 + k;
                for (int r = 0; r < R; ++r) {
                    accV[r] = fmaf(pk, dOh[ik * D + lane + r * kWave], accV[r]);
                    accK[r] = fmaf(dsk, Qh[ik * D + lane + r * kWave], accK[r]);
                }
            }
        }
    }
    for (int r = 0; r < R; ++r) {
        dK[row * D + lane + r * kWave] = p.scale * accK[r];
        dV[row * D + lane + r * kWave] = accV[r];
    }
}

unsigned blocks_for_rows(long n_rows) { return (unsigned)((n_rows + 3) / 4); }

}  // namespace

int launch_forward_fp32(const sepattn_params &p, const HeadWin &hw, const float *Q, const float *K, const float *V,
                        const int32_t *sep_idx, const int32_t *sep_prefix, const int32_t *doc_start, float *O,
                        float *LSE, hipStream_t st) {
    long n_rows = (long)p.B * p.Hq * p.L;
    dim3 grid(blocks_for_rows(n_rows)), block(256);
    if (p.d == 64)
        hipLaunchKernelGGL(fwd_fp32_kernel<64>, grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, doc_start, O, LSE, hw);
    else
        hipLaunchKernelGGL(fwd_fp32_kernel<128>, grid, block, 0, st, p, Q, K, V, sep_idx, sep_prefix, doc_start, O, LSE, hw);
    return launch_status();
}

int launch_backward_fp32(const sepattn_params &p, const HeadWin &hw, const float *Q, const float *K, const float *V,
                         const float *O, const float *LSE, const float *dO, const int32_t *sep_idx,
                         const int32_t *sep_prefix, const int32_t *doc_start, const int32_t *doc_end, float *dQ,
                         float *dK, float *dV, float *Dws, hipStream_t st) {
    long q_rows = (long)p.B * p.Hq * p.L, k_rows = (long)p.B * p.Hkv * p.L;
    dim3 block(256);
    if (p.d == 64) {
        hipLaunchKernelGGL(rowdot_fp32_kernel<64>, dim3(blocks_for_rows(q_rows)), block, 0, st, q_rows, dO, O, Dws);
        hipLaunchKernelGGL(dq_fp32_kernel<64>, dim3(blocks_for_rows(q_rows)), block, 0, st, p, Q, K, V, LSE, dO, Dws, sep_idx, sep_prefix, doc_start, dQ, hw);
        hipLaunchKernelGGL(dkv_fp32_kernel<64>, dim3(blocks_for_rows(k_rows)), block, 0, st, p, Q, K, V, LSE, dO, Dws, sep_prefix, doc_end, dK, dV, hw);
    } else {
        hipLaunchKernelGGL(rowdot_fp32_kernel<128>, dim3(blocks_for_rows(q_rows)), block, 0, st, q_rows, dO, O, Dws);
        hipLaunchKernelGGL(dq_fp32_kernel<128>, dim3(blocks_for_rows(q_rows)), block, 0, st, p, Q, K, V, LSE, dO, Dws, sep_idx, sep_prefix, doc_start, dQ, hw);
        hipLaunchKernelGGL(dkv_fp32_kernel<128>, dim3(blocks_for_rows(k_rows)), block, 0, st, p, Q, K, V, LSE, dO, Dws, sep_prefix, doc_end, dK, dV, hw);
    }
    return launch_status();
}

}  // namespace sepattn
