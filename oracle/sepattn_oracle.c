/*
 * CPU oracle for SepAttention (SepLLM, arXiv 2412.12094).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, dense implementation of what the method computes, written from the paper's
 * definitions: the explicit boolean mask M (Sec. 3.1 "Fundamental Design" and Eq. 2), dense masked
 * softmax attention (Eq. 1), the analytic gradient of Eq. 1, single-query attention over the
 * four-block KV cache and the cache compression step (Sec. 3.3 "Tailored Streaming Design").
 * No tiling, no index lists inside the attention, no fusion: every function can be checked against
 * the paper by eye.  It shares no code with the GPU library and must never be linked into or
 * called from the product path; only the tests, the smoke check and the benchmark's CPU-baseline
 * leg use it.
 *
 * Built twice from this one file: ORACLE_REAL=double (parity arbiter, finite-difference pins) and
 * ORACLE_REAL=float (the "plain CPU fp32" baseline that is timed).  Sums are always carried in
 * double.
 *
 * Readings of the paper where it is silent (also listed in the design notes):
 *   - neighbour window of query i is i-n < j <= i  (n keys, the token itself included);
 *   - initial tokens are positions 0..a-1;
 *   - a separator is a token whose id is in the caller's id set;
 *   - overlaps (a separator inside the window, ...) count once: M is a union;
 *   - grouped-query attention: query head h reads KV head h / (Hq/Hkv);
 *   - LSE is the natural log of the softmax denominator, scores include the scale;
 *   - separator-cache overflow drops the oldest entries (FIFO)           [parity unpinned];
 *   - the window region is one run in position order, oldest first: the first Size_past
 *     entries are the Past Window, the rest the Local Window             [parity unpinned].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

int oracle_real_bytes(void) { return (int)sizeof(real); }

/* ---- Sec. 4.1 "Parameter Setting": token is a separator iff its id is in the set ---------- */
void oracle_mark_separators(const int32_t *token_ids, int B, int L, const int32_t *sep_ids,
                            int n_sep, uint8_t *is_sep) {
    for (long t = 0; t < (long)B * L; ++t) {
        uint8_t f = 0;
        for (int k = 0; k < n_sep; ++k)
            if (token_ids[t] == sep_ids[k]) f = 1;
        is_sep[t] = f;
    }
}

/* ---- ascending list of separator positions, their count and the exclusive prefix count ---- */
/* sep_idx is [B, cap]; entries beyond cap are not written; sep_count holds the true count.    */
void oracle_compact_indices(const uint8_t *is_sep, int B, int L, int32_t *sep_idx, int cap,
                            int32_t *sep_count, int32_t *sep_prefix) {
    for (int b = 0; b < B; ++b) {
        int32_t cnt = 0;
        for (int j = 0; j < L; ++j) {
            if (sep_prefix) sep_prefix[(long)b * (L + 1) + j] = cnt;
            if (is_sep[(long)b * L + j]) {
                if (cnt < cap) sep_idx[(long)b * cap + cnt] = j;
                ++cnt;
            }
        }
        if (sep_prefix) sep_prefix[(long)b * (L + 1) + L] = cnt;
        sep_count[b] = cnt;
    }
}

/* ---- Sec. 3.1 + Eq. 2: M[i][j] = 1 iff key j is at or before query i and is an initial token,
 *      a separator, or one of the n closest tokens.  rows[] selects which query rows to build. */
void oracle_mask_rows(const uint8_t *is_sep /*[L]*/, int L, int a, int n, const int32_t *rows,
                      int n_rows, uint8_t *M /*[n_rows, L]*/) {
    for (int r = 0; r < n_rows; ++r) {
        int i = rows[r];
        for (int j = 0; j < L; ++j) {
            int causal = (j <= i);
            int initial = (j < a);
            int separator = is_sep[j] != 0;
            int neighbour = (i - j < n);
            M[(long)r * L + j] = (uint8_t)(causal && (initial || separator || neighbour));
        }
    }
}

/* one row of Eq. 1: Lambda_ij = scale*<Q_i,K_j> where M=1, -inf elsewhere; A = softmax(Lambda) */
static void attention_row(const real *q, const real *K, const uint8_t *m, int L, int d,
                          double scale, double *lam, double *A_row, double *lse) {
    double mx = -INFINITY;
    for (int j = 0; j < L; ++j) {
        if (m[j]) {
            double s = 0.0;
            for (int k = 0; k < d; ++k) s += (double)q[k] * (double)K[(long)j * d + k];
            lam[j] = s * scale;
            if (lam[j] > mx) mx = lam[j];
        } else {
            lam[j] = -INFINITY;
        }
    }
    double den = 0.0;
    for (int j = 0; j < L; ++j) {
        A_row[j] = m[j] ? exp(lam[j] - mx) : 0.0;
        den += A_row[j];
    }
    for (int j = 0; j < L; ++j) A_row[j] /= den;
    *lse = mx + log(den);
}

/* ---- Eq. 1 for selected rows of every (batch, head): O = A V, LSE = log sum exp(Lambda) ----
 * Q [B,Hq,L,d]; K,V [B,Hkv,L,d]; is_sep [B,L]; rows[n_rows] (NULL = all rows).
 * O [B,Hq,n_rows,d]; LSE [B,Hq,n_rows]; A_out (may be NULL) [B,Hq,n_rows,L].
 * n_head (may be NULL) [Hq]: a neighbour window of its own for every query head, in place of n
 * (the head-wise variant of Sec. 4.6 "Comparison with More Baselines and Variants": some heads keep
 * a short window, the others see everything, i.e. n_head[h] >= L); the mask of head h is then
 * Eq. 2 with n = n_head[h].                                                                     */
int oracle_forward(const real *Q, const real *K, const real *V, const uint8_t *is_sep, int B,
                   int Hq, int Hkv, int L, int d, int a, int n, const int32_t *n_head, double scale,
                   const int32_t *rows, int n_rows, real *O, real *LSE, real *A_out) {
    if (Hkv <= 0 || Hq % Hkv != 0) return 1;
    int G = Hq / Hkv;
    int32_t *all = NULL;
    if (!rows) {
        all = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
        for (int i = 0; i < L; ++i) all[i] = i;
        rows = all;
        n_rows = L;
    }
    uint8_t *M = (uint8_t *)malloc((size_t)n_rows * (size_t)L);
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            int kv = h / G;
            const real *Kh = K + ((long)b * Hkv + kv) * (long)L * d;
            const real *Vh = V + ((long)b * Hkv + kv) * (long)L * d;
            oracle_mask_rows(is_sep + (long)b * L, L, a, n_head ? n_head[h] : n, rows, n_rows, M);
#pragma omp parallel
            {
                double *lam = (double *)malloc(sizeof(double) * (size_t)L);
                double *Ar = (double *)malloc(sizeof(double) * (size_t)L);
                double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 8)
                for (int r = 0; r < n_rows; ++r) {
                    const real *q = Q + (((long)b * Hq + h) * L + rows[r]) * d;
                    double lse;
                    attention_row(q, Kh, M + (long)r * L, L, d, scale, lam, Ar, &lse);
                    for (int k = 0; k < d; ++k) o[k] = 0.0;
                    for (int j = 0; j < L; ++j) {
                        if (Ar[j] == 0.0) continue;
                        for (int k = 0; k < d; ++k) o[k] += Ar[j] * (double)Vh[(long)j * d + k];
                    }
                    long orow = ((long)b * Hq + h) * n_rows + r;
                    for (int k = 0; k < d; ++k) O[orow * d + k] = (real)o[k];
                    LSE[orow] = (real)lse;
                    if (A_out)
                        for (int j = 0; j < L; ++j) A_out[orow * L + j] = (real)Ar[j];
                }
                free(lam);
                free(Ar);
                free(o);
            }
        }
    }
    free(M);
    free(all);
    return 0;
}

/* ---- analytic gradient of Eq. 1 (the paper prints none; this is calculus on O = softmax(L)V):
 *   D_i   = sum_k dO_ik O_ik
 *   dV_j  = sum_i A_ij dO_i
 *   dA_ij = <dO_i, V_j>
 *   dL_ij = A_ij (dA_ij - D_i)            (softmax Jacobian; zero where M=0 because A=0)
 *   dQ_i  = scale sum_j dL_ij K_j,   dK_j = scale sum_i dL_ij Q_i
 * dK, dV of a KV head are summed over the Hq/Hkv query heads that read it.
 * The forward pass is recomputed densely inside (A kept as a full L x L matrix per head).
 * n_head (may be NULL) [Hq]: per-head neighbour windows, as in oracle_forward.
 *
 * eQ, eK, eV (each may be NULL; shaped like dQ, dK, dV): the root of the sum of the SQUARES of the
 * very terms that dQ, dK, dV add up,
 *   eV_jk = sqrt(sum_i (A_ij dO_ik)^2),  eK_jk = scale sqrt(sum_i (dL_ij Q_ik)^2),
 *   eQ_ik = scale sqrt(sum_j (dL_ij K_jk)^2)        (eK, eV: sums over the query heads as well).
 * They are not part of the method: an implementation that rounds every A_ij (dL_ij) to a format
 * of unit roundoff u before it adds the terms up makes an error of standard deviation at most
 * u/sqrt(3) times these numbers, which is what a parity test needs in order to state a bound for
 * gradients that are sums of thousands of terms.                                                 */
int oracle_backward(const real *Q, const real *K, const real *V, const real *dO,
                    const uint8_t *is_sep, int B, int Hq, int Hkv, int L, int d, int a, int n,
                    const int32_t *n_head, double scale, real *dQ, real *dK, real *dV, real *eQ,
                    real *eK, real *eV) {
    if (Hkv <= 0 || Hq % Hkv != 0) return 1;
    int G = Hq / Hkv;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)L);
    for (int i = 0; i < L; ++i) rows[i] = i;
    uint8_t *M = (uint8_t *)malloc((size_t)L * (size_t)L);
    double *A = (double *)malloc(sizeof(double) * (size_t)L * (size_t)L);
    double *dL = (double *)malloc(sizeof(double) * (size_t)L * (size_t)L);
    double *dKacc = (double *)malloc(sizeof(double) * (size_t)L * (size_t)d);
    double *dVacc = (double *)malloc(sizeof(double) * (size_t)L * (size_t)d);
    double *eKacc = (double *)malloc(sizeof(double) * (size_t)L * (size_t)d);
    double *eVacc = (double *)malloc(sizeof(double) * (size_t)L * (size_t)d);
    if (!M || !A || !dL || !dKacc || !dVacc || !eKacc || !eVacc) return 2;
    for (int b = 0; b < B; ++b) {
        for (int kv = 0; kv < Hkv; ++kv) {
            const real *Kh = K + ((long)b * Hkv + kv) * (long)L * d;
            const real *Vh = V + ((long)b * Hkv + kv) * (long)L * d;
            memset(dKacc, 0, sizeof(double) * (size_t)L * d);
            memset(dVacc, 0, sizeof(double) * (size_t)L * d);
            memset(eKacc, 0, sizeof(double) * (size_t)L * d);
            memset(eVacc, 0, sizeof(double) * (size_t)L * d);
            for (int g = 0; g < G; ++g) {
                int h = kv * G + g;
                const real *Qh = Q + ((long)b * Hq + h) * (long)L * d;
                const real *dOh = dO + ((long)b * Hq + h) * (long)L * d;
                real *dQh = dQ + ((long)b * Hq + h) * (long)L * d;
                real *eQh = eQ ? eQ + ((long)b * Hq + h) * (long)L * d : NULL;
                oracle_mask_rows(is_sep + (long)b * L, L, a, n_head ? n_head[h] : n, rows, L, M);
                /* forward rows, then dL rows and dQ rows */
#pragma omp parallel
                {
                    double *lam = (double *)malloc(sizeof(double) * (size_t)L);
                    double *o = (double *)malloc(sizeof(double) * (size_t)d);
                    double *dq = (double *)malloc(sizeof(double) * (size_t)d);
                    double *eq = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 8)
                    for (int i = 0; i < L; ++i) {
                        double lse;
                        double *Ai = A + (long)i * L;
                        double *dLi = dL + (long)i * L;
                        attention_row(Qh + (long)i * d, Kh, M + (long)i * L, L, d, scale, lam, Ai,
                                      &lse);
                        for (int k = 0; k < d; ++k) o[k] = 0.0;
                        for (int j = 0; j < L; ++j) {
                            if (Ai[j] == 0.0) continue;
                            for (int k = 0; k < d; ++k) o[k] += Ai[j] * (double)Vh[(long)j * d + k];
                        }
                        double D = 0.0;
                        for (int k = 0; k < d; ++k) D += (double)dOh[(long)i * d + k] * o[k];
                        for (int k = 0; k < d; ++k) dq[k] = eq[k] = 0.0;
                        for (int j = 0; j < L; ++j) {
                            if (Ai[j] == 0.0) {
                                dLi[j] = 0.0;
                                continue;
                            }
                            double dA = 0.0;
                            for (int k = 0; k < d; ++k)
                                dA += (double)dOh[(long)i * d + k] * (double)Vh[(long)j * d + k];
                            dLi[j] = Ai[j] * (dA - D);
                            for (int k = 0; k < d; ++k) {
                                double term = dLi[j] * (double)Kh[(long)j * d + k];
                                dq[k] += term;
                                eq[k] += term * term;
                            }
                        }
                        for (int k = 0; k < d; ++k) dQh[(long)i * d + k] = (real)(scale * dq[k]);
                        if (eQh)
                            for (int k = 0; k < d; ++k)
                                eQh[(long)i * d + k] = (real)(fabs(scale) * sqrt(eq[k]));
                    }
                    free(lam);
                    free(o);
                    free(dq);
                    free(eq);
                }
                /* column sums: dV_j and dK_j */
#pragma omp parallel for schedule(dynamic, 8)
                for (int j = 0; j < L; ++j) {
                    for (int i = 0; i < L; ++i) {
                        double Aij = A[(long)i * L + j];
                        if (Aij == 0.0) continue;
                        double dLij = dL[(long)i * L + j];
                        for (int k = 0; k < d; ++k) {
                            double tv = Aij * (double)dOh[(long)i * d + k];
                            double tk = scale * dLij * (double)Qh[(long)i * d + k];
                            dVacc[(long)j * d + k] += tv;
                            dKacc[(long)j * d + k] += tk;
                            eVacc[(long)j * d + k] += tv * tv;
                            eKacc[(long)j * d + k] += tk * tk;
                        }
                    }
                }
            }
            real *dKh = dK + ((long)b * Hkv + kv) * (long)L * d;
            real *dVh = dV + ((long)b * Hkv + kv) * (long)L * d;
            for (long t = 0; t < (long)L * d; ++t) {
                dKh[t] = (real)dKacc[t];
                dVh[t] = (real)dVacc[t];
            }
            if (eK)
                for (long t = 0; t < (long)L * d; ++t)
                    eK[((long)b * Hkv + kv) * (long)L * d + t] = (real)sqrt(eKacc[t]);
            if (eV)
                for (long t = 0; t < (long)L * d; ++t)
                    eV[((long)b * Hkv + kv) * (long)L * d + t] = (real)sqrt(eVacc[t]);
        }
    }
    free(rows);
    free(M);
    free(A);
    free(dL);
    free(dKacc);
    free(dVacc);
    free(eKacc);
    free(eVacc);
    return 0;
}

/* ---- Sec. 3.2 "Generation" / Sec. 3.3: one query per sequence over every valid cache entry ---
 * Cache layout per (sequence, KV head): c slots of d values:
 *   [0,a) Initial | [a,a+s) Separator | [a+s,c) window (Past Window then Local Window, oldest
 *   first).  sizes[S,4] = (Size_init, Size_sep, Size_past_w, Size_local_w).
 * All valid entries are visible, so this is Eq. 1 with a single query row and M = 1.             */
int oracle_decode(const real *q /*[S,Hq,d]*/, const real *Kc, const real *Vc /*[S,Hkv,c,d]*/,
                  const int32_t *sizes, int S, int Hq, int Hkv, int d, int a, int s, int c,
                  double scale, real *out /*[S,Hq,d]*/, real *lse /*[S,Hq] or NULL*/) {
    if (Hkv <= 0 || Hq % Hkv != 0) return 1;
    int G = Hq / Hkv;
    for (int sq = 0; sq < S; ++sq) {
        const int32_t *sz = sizes + 4 * sq;
        if (sz[0] < 0 || sz[0] > a || sz[1] < 0 || sz[1] > s || sz[2] < 0 || sz[3] < 0 ||
            sz[2] + sz[3] > c - a - s)
            return 3;
        int n_valid = sz[0] + sz[1] + sz[2] + sz[3];
        if (n_valid == 0) return 4;
        int32_t *slots = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_valid);
        int t = 0;
        for (int k = 0; k < sz[0]; ++k) slots[t++] = k;
        for (int k = 0; k < sz[1]; ++k) slots[t++] = a + k;
        for (int k = 0; k < sz[2] + sz[3]; ++k) slots[t++] = a + s + k;
        real *Kg = (real *)malloc(sizeof(real) * (size_t)n_valid * d);
        uint8_t *ones = (uint8_t *)malloc((size_t)n_valid);
        double *lam = (double *)malloc(sizeof(double) * (size_t)n_valid);
        double *Ar = (double *)malloc(sizeof(double) * (size_t)n_valid);
        memset(ones, 1, (size_t)n_valid);
        for (int h = 0; h < Hq; ++h) {
            int kv = h / G;
            const real *Kh = Kc + ((long)sq * Hkv + kv) * (long)c * d;
            const real *Vh = Vc + ((long)sq * Hkv + kv) * (long)c * d;
            for (int e = 0; e < n_valid; ++e)
                memcpy(Kg + (long)e * d, Kh + (long)slots[e] * d, sizeof(real) * (size_t)d);
            double l;
            attention_row(q + ((long)sq * Hq + h) * d, Kg, ones, n_valid, d, scale, lam, Ar, &l);
            for (int k = 0; k < d; ++k) {
                double o = 0.0;
                for (int e = 0; e < n_valid; ++e) o += Ar[e] * (double)Vh[(long)slots[e] * d + k];
                out[((long)sq * Hq + h) * d + k] = (real)o;
            }
            if (lse) lse[(long)sq * Hq + h] = (real)l;
        }
        free(slots);
        free(Kg);
        free(ones);
        free(lam);
        free(Ar);
    }
    return 0;
}

/* ---- Sec. 3.3, compression step (Fig. "streaming design" caption): separators of the Past
 * Window move to the Separator Cache, the other Past-Window entries are dropped; the Local
 * Window becomes the whole window.  Rows are raw bytes (row_bytes each) and are copied exactly.
 * Kc, Vc [S,Hkv,c,row]; win_is_sep [S, c-a-s]; sizes [S,4]; everything updated in place.
 * If the Separator Cache would overflow its capacity s, its oldest entries are dropped.          */
int oracle_evict_window(uint8_t *Kc, uint8_t *Vc, uint8_t *win_is_sep, int32_t *sizes, int S,
                        int Hkv, int a, int s, int c, long row_bytes) {
    int wcap = c - a - s;
    if (wcap <= 0) return 1;
    for (int sq = 0; sq < S; ++sq) {
        int32_t *sz = sizes + 4 * sq;
        int P = sz[2], Lw = sz[3], Ns = sz[1];
        if (P < 0 || Lw < 0 || P + Lw > wcap || Ns < 0 || Ns > s) return 3;
        uint8_t *fl = win_is_sep + (long)sq * wcap;
        /* the new separator list: old entries, then flagged Past-Window entries, oldest first */
        int total = Ns;
        for (int t = 0; t < P; ++t) total += fl[t] ? 1 : 0;
        int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
        int m = 0;
        for (int k = 0; k < Ns; ++k) src[m++] = a + k;
        for (int t = 0; t < P; ++t)
            if (fl[t]) src[m++] = a + s + t;
        int drop = total > s ? total - s : 0;
        int Ns_new = total - drop;
        for (int kv = 0; kv < Hkv; ++kv) {
            for (int which = 0; which < 2; ++which) {
                uint8_t *base = (which ? Vc : Kc) + ((long)sq * Hkv + kv) * (long)c * row_bytes;
                uint8_t *old = (uint8_t *)malloc((size_t)c * (size_t)row_bytes);
                memcpy(old, base, (size_t)c * (size_t)row_bytes);
                for (int k = 0; k < Ns_new; ++k)
                    memcpy(base + (long)(a + k) * row_bytes, old + (long)src[drop + k] * row_bytes,
                           (size_t)row_bytes);
                for (int t = 0; t < Lw; ++t)
                    memcpy(base + (long)(a + s + t) * row_bytes,
                           old + (long)(a + s + P + t) * row_bytes, (size_t)row_bytes);
                free(old);
            }
        }
        for (int t = 0; t < Lw; ++t) fl[t] = fl[P + t];
        sz[1] = Ns_new;
        sz[2] = 0;
        sz[3] = Lw;
        free(src);
    }
    return 0;
}
