/*
 * CPU oracle for the AnTKV online path.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product (the HIP library and its Python binding) may call, link or import it.
 *
 * Every function is the plain definition written out in fp64, one output element
 * at a time, with no blocking, fusion or reordering beyond OpenMP over
 * independent outputs.  Inputs that are fp16 in the method arrive here as fp32
 * arrays holding exactly the fp16 values (the widening fp16 -> fp32 is exact).
 *
 *   oracle_encode          nearest-centroid assignment of sub-vectors
 *                          (paper Sec. 3.1: token rows are split into sub-vectors
 *                          and replaced by k-means centroids).
 *   oracle_anchor_score    Anchor Score of every key position, Eq. (4):
 *                          AnS(V_j) = sum_i A_ij,
 *                          AnS(K_j) = sum_i A_ij (1 - A_ij) ||Q_i||_2,
 *                          A = causal softmax(scale * Q K^T), summed over the query
 *                          heads that share a KV head.
 *   oracle_decode_attn     Attn(q, K_eff, V_eff) (Sec. 2.1) where row j of K_eff /
 *                          V_eff is the FP16 anchor row if j is an anchor and the
 *                          concatenation of the coded centroids otherwise (Sec. 3,
 *                          Fig. 2(b)); optionally also Eq. (4) for the single
 *                          decode query over K_eff.
 *
 * Parity status: all three functions are pinned by tests/test_oracle_*.py against
 * library routines, closed forms and the equality case of the paper's Eq. (3).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- *
 * Encode.  x: [B][Hkv][n][D], cb: [Hkv][M][C][d] with M = D/d.
 * codes: [B][Hkv][n][M] (int32 so that any C fits).
 * margin (optional): (second smallest distance - smallest) /
 *                    max(||x_m||^2 + ||cb[code]||^2, 1e-30)
 * Ties resolve to the lower centroid index.
 * ------------------------------------------------------------------------- */
int oracle_encode(const float *x, const float *cb, int64_t B, int64_t Hkv, int64_t n,
                  int64_t D, int64_t d, int64_t C, int32_t *codes, double *margin)
{
    if (d <= 0 || D % d != 0 || C < 1) return -1;
    const int64_t M = D / d;
    const int64_t rows = B * Hkv * n;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t g = (r / n) % Hkv;
        const float *xr = x + r * D;
        for (int64_t m = 0; m < M; ++m) {
            const float *xs = xr + m * d;
            const float *tab = cb + ((g * M + m) * C) * d;
            double best = INFINITY, second = INFINITY;
            int64_t bi = -1;
            for (int64_t c = 0; c < C; ++c) {
                double dist = 0.0;
                for (int64_t t = 0; t < d; ++t) {
                    const double diff = (double)xs[t] - (double)tab[c * d + t];
                    dist += diff * diff;
                }
                if (dist < best) {
                    second = best;
                    best = dist;
                    bi = c;
                } else if (dist < second) {
                    second = dist;
                }
            }
            codes[r * M + m] = (int32_t)bi;
            if (margin) {
                double nx = 0.0, nc = 0.0;
                for (int64_t t = 0; t < d; ++t) {
                    nx += (double)xs[t] * (double)xs[t];
                    nc += (double)tab[bi * d + t] * (double)tab[bi * d + t];
                }
                const double den = fmax(nx + nc, 1e-30);
                margin[r * M + m] = (C > 1) ? (second - best) / den : INFINITY;
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- *
 * Anchor Score, Eq. (4).  q: [B][Hq][Nq][D], k: [B][Hkv][N][D].
 * Query row i sits at absolute position N - Nq + i and (if causal) sees keys
 * 0..N-Nq+i.  Outputs ans_k, ans_v: [B][Hkv][N], the sum over the Hq/Hkv query
 * heads of each KV head (head h reads KV head h / (Hq/Hkv)).
 * Optional row statistics (any may be NULL), each [B][Hq][Nq]:
 *   row_max[i] = max_j S_ij, row_sum[i] = sum_j exp(S_ij - row_max[i]),
 *   q_norm[i]  = ||Q_i||_2      (the three auxiliary tensors of Sec. 3.3).
 * ------------------------------------------------------------------------- */
int oracle_anchor_score(const float *q, const float *k, int64_t B, int64_t Hq, int64_t Hkv,
                        int64_t N, int64_t Nq, int64_t D, double scale, int causal,
                        double *ans_k, double *ans_v,
                        double *row_max, double *row_sum, double *q_norm)
{
    if (Hq % Hkv != 0 || Nq > N || Nq < 0) return -1;
    const int64_t G = Hq / Hkv;
    const int64_t units = B * Hq;
    /* one accumulator pair per (b, query head); summed over heads afterwards in
       fixed order so the result does not depend on the thread schedule */
    double *acc_k = (double *)calloc((size_t)(units * N), sizeof(double));
    double *acc_v = (double *)calloc((size_t)(units * N), sizeof(double));
    if ((!acc_k || !acc_v) && units * N > 0) {
        free(acc_k);
        free(acc_v);
        return -2;
    }
    int fail = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)(N > 0 ? N : 1) * sizeof(double));
        double *qd = (double *)malloc((size_t)D * sizeof(double));
        if (!s || !qd) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t u = 0; u < units; ++u) {
            /* one thread owns all query rows of a (b, head) unit, so acc needs no
               atomics and the summation order over i is fixed */
            for (int64_t i = 0; i < Nq; ++i) {
                if (!s || !qd) continue;
                const int64_t b = u / Hq, h = u % Hq, g = h / G;
                const float *qr = q + ((b * Hq + h) * Nq + i) * D;
                const float *kb = k + ((b * Hkv + g) * N) * D;
                const int64_t last = causal ? (N - Nq + i) : (N - 1); /* last visible key */
                double nq2 = 0.0;
                for (int64_t t = 0; t < D; ++t) {
                    qd[t] = (double)qr[t];
                    nq2 += qd[t] * qd[t];
                }
                const double nq = sqrt(nq2);
                double mx = -INFINITY;
                for (int64_t j = 0; j <= last; ++j) {
                    const float *kr = kb + j * D;
                    double dot = 0.0;
#pragma omp simd reduction(+ : dot)
                    for (int64_t t = 0; t < D; ++t) dot += qd[t] * (double)kr[t];
                    s[j] = scale * dot;
                    if (s[j] > mx) mx = s[j];
                }
                double sum = 0.0;
                for (int64_t j = 0; j <= last; ++j) {
                    s[j] = exp(s[j] - mx);
                    sum += s[j];
                }
                double *ak = acc_k + u * N, *av = acc_v + u * N;
                for (int64_t j = 0; j <= last; ++j) {
                    const double a = s[j] / sum;
                    av[j] += a;
                    ak[j] += a * (1.0 - a) * nq;
                }
                const int64_t ri = (b * Hq + h) * Nq + i;
                if (row_max) row_max[ri] = mx;
                if (row_sum) row_sum[ri] = sum;
                if (q_norm) q_norm[ri] = nq;
            }
        }
        free(s);
        free(qd);
    }
    if (!fail) {
        for (int64_t b = 0; b < B; ++b)
            for (int64_t g = 0; g < Hkv; ++g)
                for (int64_t j = 0; j < N; ++j) {
                    double sk = 0.0, sv = 0.0;
                    for (int64_t hh = 0; hh < G; ++hh) {
                        const int64_t u = b * Hq + g * G + hh;
                        sk += acc_k[u * N + j];
                        sv += acc_v[u * N + j];
                    }
                    ans_k[(b * Hkv + g) * N + j] = sk;
                    ans_v[(b * Hkv + g) * N + j] = sv;
                }
    }
    free(acc_k);
    free(acc_v);
    return fail ? -2 : 0;
}

/* ------------------------------------------------------------------------- *
 * Decode attention over VQ codes + FP16 anchors.
 *   q:        [B][Hq][D]
 *   codes_k/v:[B][Hkv][N][M] int32, cb_k/v: [Hkv][M][C][d]
 *   idx_k:    [B][Hkv][k_k] int32 (unique, in [0,N)), rows_k: [B][Hkv][k_k][D]
 *   idx_v, rows_v likewise with k_v.
 * Row j of K_eff is rows_k[slot] if j == idx_k[slot] else the concatenated
 * centroids cb_k[g][m][codes_k[j][m]]; V_eff likewise.
 *   out:      [B][Hq][D] fp64 = softmax(scale * q K_eff^T) V_eff
 * Optional (may be NULL): lse [B][Hq] = log(sum_j exp(s_j)); ans_k, ans_v
 * [B][Hkv][N] = Eq. (4) for the single query row over K_eff.
 * ------------------------------------------------------------------------- */
int oracle_decode_attn(const float *q, const int32_t *codes_k, const int32_t *codes_v,
                       const float *cb_k, const float *cb_v,
                       const int32_t *idx_k, const float *rows_k, int64_t k_k,
                       const int32_t *idx_v, const float *rows_v, int64_t k_v,
                       int64_t B, int64_t Hq, int64_t Hkv, int64_t N, int64_t D, int64_t d,
                       int64_t C, double scale, double *out, double *lse,
                       double *ans_k, double *ans_v)
{
    if (Hq % Hkv != 0 || d <= 0 || D % d != 0) return -1;
    const int64_t G = Hq / Hkv, M = D / d;
    for (int64_t i = 0; i < B * Hkv * k_k; ++i)
        if (idx_k[i] < 0 || idx_k[i] >= N) return -3;
    for (int64_t i = 0; i < B * Hkv * k_v; ++i)
        if (idx_v[i] < 0 || idx_v[i] >= N) return -3;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bg = 0; bg < B * Hkv; ++bg) {
        const int64_t b = bg / Hkv, g = bg % Hkv;
        int32_t *slot_k = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
        int32_t *slot_v = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
        double *p = (double *)malloc((size_t)(N > 0 ? N : 1) * G * sizeof(double));
        double *row = (double *)malloc((size_t)D * sizeof(double));
        if (!slot_k || !slot_v || !p || !row) {
#pragma omp atomic write
            fail = 1;
            free(slot_k); free(slot_v); free(p); free(row);
            continue;
        }
        for (int64_t j = 0; j < N; ++j) slot_k[j] = slot_v[j] = -1;
        for (int64_t i = 0; i < k_k; ++i) slot_k[idx_k[bg * k_k + i]] = (int32_t)i;
        for (int64_t i = 0; i < k_v; ++i) slot_v[idx_v[bg * k_v + i]] = (int32_t)i;

        /* scores s[hh][j] = scale * q_h . K_eff[j] */
        for (int64_t j = 0; j < N; ++j) {
            if (slot_k[j] >= 0) {
                const float *r = rows_k + (bg * k_k + slot_k[j]) * D;
                for (int64_t t = 0; t < D; ++t) row[t] = (double)r[t];
            } else {
                for (int64_t m = 0; m < M; ++m) {
                    const int64_t c = codes_k[(bg * N + j) * M + m];
                    const float *cen = cb_k + ((g * M + m) * C + c) * d;
                    for (int64_t t = 0; t < d; ++t) row[m * d + t] = (double)cen[t];
                }
            }
            for (int64_t hh = 0; hh < G; ++hh) {
                const float *qr = q + (b * Hq + g * G + hh) * D;
                double dot = 0.0;
                for (int64_t t = 0; t < D; ++t) dot += (double)qr[t] * row[t];
                p[hh * N + j] = scale * dot;
            }
        }
        /* softmax per head */
        for (int64_t hh = 0; hh < G; ++hh) {
            double mx = -INFINITY, sum = 0.0;
            for (int64_t j = 0; j < N; ++j)
                if (p[hh * N + j] > mx) mx = p[hh * N + j];
            for (int64_t j = 0; j < N; ++j) {
                p[hh * N + j] = exp(p[hh * N + j] - mx);
                sum += p[hh * N + j];
            }
            for (int64_t j = 0; j < N; ++j) p[hh * N + j] /= sum;
            if (lse) lse[b * Hq + g * G + hh] = (N > 0) ? mx + log(sum) : -INFINITY;
        }
        /* out = sum_j p_j V_eff[j] */
        for (int64_t hh = 0; hh < G; ++hh)
            for (int64_t t = 0; t < D; ++t) out[(b * Hq + g * G + hh) * D + t] = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            if (slot_v[j] >= 0) {
                const float *r = rows_v + (bg * k_v + slot_v[j]) * D;
                for (int64_t t = 0; t < D; ++t) row[t] = (double)r[t];
            } else {
                for (int64_t m = 0; m < M; ++m) {
                    const int64_t c = codes_v[(bg * N + j) * M + m];
                    const float *cen = cb_v + ((g * M + m) * C + c) * d;
                    for (int64_t t = 0; t < d; ++t) row[m * d + t] = (double)cen[t];
                }
            }
            for (int64_t hh = 0; hh < G; ++hh) {
                const double pj = p[hh * N + j];
                double *o = out + (b * Hq + g * G + hh) * D;
                for (int64_t t = 0; t < D; ++t) o[t] += pj * row[t];
            }
        }
        /* decode-time Anchor Score: Eq. (4) with the one query row */
        if (ans_k || ans_v) {
            for (int64_t j = 0; j < N; ++j) {
                double sk = 0.0, sv = 0.0;
                for (int64_t hh = 0; hh < G; ++hh) {
                    const float *qr = q + (b * Hq + g * G + hh) * D;
                    double n2 = 0.0;
                    for (int64_t t = 0; t < D; ++t) n2 += (double)qr[t] * (double)qr[t];
                    const double a = p[hh * N + j];
                    sv += a;
                    sk += a * (1.0 - a) * sqrt(n2);
                }
                if (ans_k) ans_k[bg * N + j] = sk;
                if (ans_v) ans_v[bg * N + j] = sv;
            }
        }
        free(slot_k); free(slot_v); free(p); free(row);
    }
    return fail ? -2 : 0;
}
