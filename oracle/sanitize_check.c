/* Host-only check of the C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (TEST INFRASTRUCTURE, like
 * the oracle itself): calls every entry point of antkv_oracle.c on small ragged shapes, with and without the optional
 * outputs, with empty anchor lists and with lists that cover every token.  Built and run by
 * tests/test_oracle_sanitizers.py; a sanitizer report aborts the program. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_encode(const float *x, const float *cb, int64_t B, int64_t Hkv, int64_t n, int64_t D, int64_t d, int64_t C,
                  int32_t *codes, double *margin);
int oracle_anchor_score(const float *q, const float *k, int64_t B, int64_t Hq, int64_t Hkv, int64_t N, int64_t Nq,
                        int64_t D, double scale, int causal, double *ans_k, double *ans_v, double *row_max,
                        double *row_sum, double *q_norm);
int oracle_decode_attn(const float *q, const int32_t *codes_k, const int32_t *codes_v, const float *cb_k,
                       const float *cb_v, const int32_t *idx_k, const float *rows_k, int64_t k_k, const int32_t *idx_v,
                       const float *rows_v, int64_t k_v, int64_t B, int64_t Hq, int64_t Hkv, int64_t N, int64_t D,
                       int64_t d, int64_t C, double scale, double *out, double *lse, double *ans_k, double *ans_v);

static uint64_t state = 88172645463325252ull;
static double rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}
static float *fl(int64_t n)
{
    float *p = malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));   /* exact sizes: an overrun by one element is caught */
    if (n > 0) p = realloc(p, sizeof(float) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) p[i] = (float)(4.0 * rnd());
    return p;
}
static double *db(int64_t n) { return malloc(sizeof(double) * (size_t)(n > 0 ? n : 1)); }

static int run(int64_t B, int64_t Hq, int64_t Hkv, int64_t N, int64_t Nq, int64_t D, int64_t d, int64_t C, int64_t k_k,
               int64_t k_v)
{
    const int64_t M = D / d;
    int rc = 0;
    float *x = fl(B * Hkv * N * D), *cbk = fl(Hkv * M * C * d), *cbv = fl(Hkv * M * C * d);
    int32_t *ck = malloc(sizeof(int32_t) * (size_t)(B * Hkv * N * M + 1)), *cv = malloc(sizeof(int32_t) * (size_t)(B * Hkv * N * M + 1));
    double *margin = db(B * Hkv * N * M);
    rc |= oracle_encode(x, cbk, B, Hkv, N, D, d, C, ck, margin);
    rc |= oracle_encode(x, cbv, B, Hkv, N, D, d, C, cv, NULL);
    float *qw = fl(B * Hq * Nq * D);
    double *ak = db(B * Hkv * N), *av = db(B * Hkv * N), *rm = db(B * Hq * Nq), *rs = db(B * Hq * Nq), *qn = db(B * Hq * Nq);
    rc |= oracle_anchor_score(qw, x, B, Hq, Hkv, N, Nq, D, 0.3, 1, ak, av, rm, rs, qn);
    rc |= oracle_anchor_score(qw, x, B, Hq, Hkv, N, Nq, D, 0.3, 0, ak, av, NULL, NULL, NULL);
    /* ascending anchor lists: evenly spread positions */
    int32_t *ik = malloc(sizeof(int32_t) * (size_t)(B * Hkv * k_k + 1)), *iv = malloc(sizeof(int32_t) * (size_t)(B * Hkv * k_v + 1));
    for (int64_t r = 0; r < B * Hkv; ++r) {
        for (int64_t i = 0; i < k_k; ++i) ik[r * k_k + i] = (int32_t)(i * N / k_k);
        for (int64_t i = 0; i < k_v; ++i) iv[r * k_v + i] = (int32_t)(N - 1 - (k_v - 1 - i) * N / k_v);
    }
    float *rk = fl(B * Hkv * k_k * D), *rv = fl(B * Hkv * k_v * D), *q = fl(B * Hq * D);
    double *out = db(B * Hq * D), *lse = db(B * Hq);
    rc |= oracle_decode_attn(q, ck, cv, cbk, cbv, ik, rk, k_k, iv, rv, k_v, B, Hq, Hkv, N, D, d, C, 0.2, out, lse, ak, av);
    rc |= oracle_decode_attn(q, ck, cv, cbk, cbv, ik, rk, k_k, iv, rv, k_v, B, Hq, Hkv, N, D, d, C, 0.2, out, NULL, NULL, NULL);
    free(x); free(cbk); free(cbv); free(ck); free(cv); free(margin); free(qw); free(ak); free(av); free(rm); free(rs);
    free(qn); free(ik); free(iv); free(rk); free(rv); free(q); free(out); free(lse);
    return rc;
}

int main(void)
{
    int rc = 0;
    rc |= run(2, 4, 2, 37, 37, 16, 4, 256, 3, 5);       /* ragged sizes, a full query window */
    rc |= run(1, 8, 2, 130, 9, 128, 8, 256, 0, 0);      /* the real head dimension, no anchors */
    rc |= run(1, 2, 1, 5, 1, 32, 16, 7, 5, 5);          /* every token anchored in both lists, a tiny odd codebook */
    rc |= run(1, 4, 4, 1, 1, 128, 32, 4096, 1, 0);      /* one token, 4096 centroids */
    rc |= run(3, 6, 3, 64, 64, 8, 8, 2, 1, 64);         /* one sub-space */
    printf(rc == 0 ? "sanitize_check: ok\n" : "sanitize_check: an oracle call returned an error\n");
    return rc != 0;
}
