/* Memory-safety check of the C oracle (TEST INFRASTRUCTURE ONLY): runs every oracle function on a
 * few small, ragged and degenerate shapes.  Built by tests/test_oracle_sanitizers.py with
 * -fsanitize=address,undefined (exact-size heap buffers, so that any read or write beyond an
 * operand trips the sanitizer) and run on the CPU; it prints one line and returns 0.            */
#include "sepattn_oracle.c"

#include <stdio.h>

static unsigned long long state = 0x5E9A77ULL;
static double rnd(void) {
    state = state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static real *vec(long n) {
    real *p = (real *)malloc(sizeof(real) * (size_t)(n > 0 ? n : 1));
    for (long i = 0; i < n; ++i) p[i] = (real)rnd();
    return p;
}

static int attention_case(int B, int Hq, int Hkv, int L, int d, int a, int n, double p_sep, int cap) {
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * L);
    const int32_t ids[3] = {11, 13, 198};
    for (long t = 0; t < (long)B * L; ++t) tok[t] = rnd() + 0.5 < p_sep ? ids[t % 3] : 1000 + (int32_t)(t % 7);
    uint8_t *is_sep = (uint8_t *)malloc((size_t)B * L);
    oracle_mark_separators(tok, B, L, ids, 3, is_sep);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * cap);
    int32_t *cnt = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
    int32_t *pre = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * (L + 1));
    oracle_compact_indices(is_sep, B, L, idx, cap, cnt, pre);
    oracle_compact_indices(is_sep, B, L, idx, cap, cnt, NULL);
    real *Q = vec((long)B * Hq * L * d), *K = vec((long)B * Hkv * L * d), *V = vec((long)B * Hkv * L * d);
    real *dO = vec((long)B * Hq * L * d);
    real *O = vec((long)B * Hq * L * d), *LSE = vec((long)B * Hq * L), *A = vec((long)B * Hq * L * L);
    int rc = oracle_forward(Q, K, V, is_sep, B, Hq, Hkv, L, d, a, n, NULL, 0.3, NULL, 0, O, LSE, A);
    /* a subset of rows, last row included */
    int32_t rows[2] = {0, L - 1};
    real *O2 = vec((long)B * Hq * 2 * d), *L2 = vec((long)B * Hq * 2);
    rc |= oracle_forward(Q, K, V, is_sep, B, Hq, Hkv, L, d, a, n, NULL, 0.3, rows, 2, O2, L2, NULL);
    real *dQ = vec((long)B * Hq * L * d), *dK = vec((long)B * Hkv * L * d), *dV = vec((long)B * Hkv * L * d);
    rc |= oracle_backward(Q, K, V, dO, is_sep, B, Hq, Hkv, L, d, a, n, NULL, 0.3, dQ, dK, dV, NULL, NULL, NULL);
    /* per-head windows and the term-magnitude outputs */
    int32_t *nh = (int32_t *)malloc(sizeof(int32_t) * (size_t)Hq);
    for (int h = 0; h < Hq; ++h) nh[h] = h % 2 ? L + 5 : 1 + h;
    real *eQ = vec((long)B * Hq * L * d), *eK = vec((long)B * Hkv * L * d), *eV = vec((long)B * Hkv * L * d);
    rc |= oracle_forward(Q, K, V, is_sep, B, Hq, Hkv, L, d, a, n, nh, 0.3, NULL, 0, O, LSE, NULL);
    rc |= oracle_backward(Q, K, V, dO, is_sep, B, Hq, Hkv, L, d, a, n, nh, 0.3, dQ, dK, dV, eQ, eK, eV);
    free(nh); free(eQ); free(eK); free(eV);
    double chk = 0;
    for (long i = 0; i < (long)B * Hq * L * d; ++i) chk += O[i] + dQ[i];
    free(tok); free(is_sep); free(idx); free(cnt); free(pre); free(Q); free(K); free(V); free(dO);
    free(O); free(LSE); free(A); free(O2); free(L2); free(dQ); free(dK); free(dV);
    return rc || !(chk == chk);
}

static int cache_case(int S, int Hq, int Hkv, int d, int a, int s, int c, const int32_t *sizes_in) {
    const int wcap = c - a - s;
    real *q = vec((long)S * Hq * d), *Kc = vec((long)S * Hkv * c * d), *Vc = vec((long)S * Hkv * c * d);
    real *out = vec((long)S * Hq * d), *lse = vec((long)S * Hq);
    int32_t *sizes = (int32_t *)malloc(sizeof(int32_t) * 4 * (size_t)S);
    memcpy(sizes, sizes_in, sizeof(int32_t) * 4 * (size_t)S);
    int rc = oracle_decode(q, Kc, Vc, sizes, S, Hq, Hkv, d, a, s, c, 0.2, out, lse);
    rc |= oracle_decode(q, Kc, Vc, sizes, S, Hq, Hkv, d, a, s, c, 0.2, out, NULL);
    uint8_t *flags = (uint8_t *)malloc((size_t)S * wcap);
    for (long i = 0; i < (long)S * wcap; ++i) flags[i] = rnd() > 0.1;  /* most entries flagged: overflow */
    rc |= oracle_evict_window((uint8_t *)Kc, (uint8_t *)Vc, flags, sizes, S, Hkv, a, s, c, (long)(d * sizeof(real)));
    rc |= oracle_decode(q, Kc, Vc, sizes, S, Hq, Hkv, d, a, s, c, 0.2, out, lse);
    free(q); free(Kc); free(Vc); free(out); free(lse); free(sizes); free(flags);
    return rc;
}

int main(void) {
    int bad = 0;
    bad |= attention_case(1, 1, 1, 1, 4, 4, 64, 0.0, 1);     /* a single token                      */
    bad |= attention_case(2, 4, 2, 37, 8, 3, 5, 0.2, 37);    /* ragged, GQA                         */
    bad |= attention_case(1, 2, 1, 19, 4, 50, 1, 1.0, 4);    /* a >= L, n = 1, capacity < count     */
    bad |= attention_case(1, 3, 3, 23, 4, 0, 1000, 0.0, 1);  /* a = 0, window beyond the sequence   */
    const int32_t sz1[8] = {2, 3, 4, 2, 0, 0, 0, 1};         /* one ordinary sequence, one with a single entry */
    bad |= cache_case(2, 4, 2, 4, 2, 3, 12, sz1);
    const int32_t sz2[4] = {1, 5, 6, 3};                     /* separator cache full: overflow      */
    bad |= cache_case(1, 2, 1, 8, 1, 5, 15, sz2);
    printf("oracle sanitize check: %s\n", bad ? "FAILED" : "ok");
    return bad;
}
