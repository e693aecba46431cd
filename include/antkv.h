/*
 * antkv.h - C ABI of the AnTKV online path on AMD MI355X (gfx950).
 *
 * AnTKV (Anchor Token-Aware Sub-Bit Vector Quantization for KV Cache) keeps the KV
 * cache as vector-quantization codes and preserves a small set of "anchor" tokens
 * in FP16.  This library holds the online stage (paper Sec. 3, Fig. 2(b)):
 *
 *   antkv_encode         VQ assignment of K / V sub-vectors            (Sec. 3.1)
 *   antkv_kmeans_step    one iteration of the offline token-weighted k-means (Sec. 3.1)
 *   antkv_prefill_attn   causal prompt attention + softmax row stats   (Sec. 2.1; Sec. 3.3, Alg. 1 first step)
 *   antkv_anchor_select  Anchor Score of every token + top-k select    (Sec. 3.2, Eq. (4); Sec. 3.3, Alg. 1)
 *   antkv_topk           the selection step alone
 *   antkv_gather_rows    copy the selected FP16 rows into the anchor store
 *   antkv_decode_attn    decode attention over codes + FP16 anchors    (Sec. 2.1 Attn; Sec. 3.2 last par.)
 *   antkv_decode_attn_static   the same with scratch inside the library, for callers that cannot allocate
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless stated otherwise.  The caller owns all
 *     buffers; the library never allocates, frees or synchronises.  Scratch memory is
 *     a caller-provided workspace whose size comes from the *_workspace query
 *     (256-byte aligned); antkv_decode_attn_static alone uses an array inside the library
 *     instead.  Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).
 *   - Every call returns an int: ANTKV_OK or one of the error codes below.  Argument
 *     errors are detected on the host before anything is enqueued.
 *   - Tensors are dense, row-major, last index fastest, in the layouts given per call.
 *     fp16 = IEEE binary16.  "KV head g of query head h" is g = h / (Hq / Hkv).
 *   - Geometry: D must be 128 and Hq / Hkv in {1, 2, 4}; M = D / d_sub sub-spaces per head.  Two code formats:
 *       n_centroids 256, d_sub in {4, 8, 16}: one byte per code (2 / 1 / 0.5 bit per element, the paper's
 *         d4m256 / d8m256 notation, Sec. 4); every entry point supports it.
 *       n_centroids 4096, d_sub 32 or 16: 12-bit codes (0.375 / 0.75 bit per element, the d32m4096 and d16m4096
 *         points of Sec. 4); every entry point that touches codes supports it.
 *   - Codebooks: fp16 [Hkv][M][n_centroids][d_sub], separate for K and V; sub-space m covers
 *     channels [m*d_sub, (m+1)*d_sub).
 *   - Codes: uint8 [B][Hkv][N_cap][code_bytes], token-major.  code_bytes = M for one-byte codes.  For 12-bit
 *     codes code_bytes = 3 M / 2 (6 for d_sub 32, 12 for d_sub 16): the token's M codes packed little-endian,
 *     code m at bits 12 m .. 12 m + 11 of the row (c0 | c1 << 12 | c2 << 24 | c3 << 36 for each six bytes).
 *   - Calls that share a workspace must not overlap in time.  A workspace may hold any bytes when it is first
 *     used (nothing has to be cleared) and may be reused by calls of different shapes.
 *   - Codes and index sets are deterministic.  The fp16 output of antkv_decode_attn can differ between two runs
 *     in its last bits (work is handed to wavefronts dynamically, so the order of the fp32 partial sums varies).
 */
#ifndef ANTKV_H
#define ANTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANTKV_OK 0
#define ANTKV_EINVAL 1       /* null pointer, bad shape, misaligned pointer, k out of range */
#define ANTKV_EUNSUPPORTED 2 /* geometry outside the supported set */
#define ANTKV_EWORKSPACE 3   /* workspace missing or too small */
#define ANTKV_ELAUNCH 4      /* a HIP call failed while enqueueing */

typedef struct antkv_geom {
    int32_t B;           /* sequences in the batch */
    int32_t Hq;          /* query heads */
    int32_t Hkv;         /* KV heads */
    int32_t D;           /* head dim (128) */
    int32_t d_sub;       /* sub-vector dim: 4, 8 or 16 (with 256 centroids), or 32 or 16 (with 4096) */
    int32_t n_centroids; /* 256 or 4096 */
} antkv_geom;

int antkv_version(void);
const char* antkv_strerror(int code); /* host pointer to a static string */

/*
 * VQ encode (Sec. 3.1: each token row is split into sub-vectors and each sub-vector is
 * replaced by the index of its k-means centroid, i.e. the Euclidean-nearest one).
 *
 *   x        fp16 [B][Hkv][n_tok][D] with element strides xs_b, xs_h, xs_t (channel stride 1);
 *            16-byte aligned, strides multiples of 8 elements.
 *   codebook fp16 [Hkv][M][n_centroids][d_sub]
 *   codes    uint8 [B][Hkv][N_cap][code_bytes]; rows token_offset .. token_offset+n_tok-1 are written:
 *            codes[b][g][token_offset+t][m] = argmin_c || x[b][g][t][m*d_sub : (m+1)*d_sub] - codebook[g][m][c] ||^2,
 *            the lowest c among equal distances (distances compared in fp32).
 *            With 256 centroids the squared norm of a centroid's sub-vector must stay below 2.09e6 (its half is held
 *            in fp16 terms scaled by 16); larger centroids are never chosen.  No such limit with 4096 centroids.
 * Call once for K with the K codebook and once for V with the V codebook.
 * n_tok == 0 is a no-op.  Errors: EINVAL (null, alignment, token_offset + n_tok > N_cap), EUNSUPPORTED.
 */
int antkv_encode(const antkv_geom* geom, const void* x, int64_t xs_b, int64_t xs_h, int64_t xs_t,
                 int64_t n_tok, const void* codebook, uint8_t* codes, int64_t N_cap,
                 int64_t token_offset, void* stream);

/*
 * Anchor Score + selection (Eq. (4)):
 *   AnS(V_j) = sum_i A_ij,   AnS(K_j) = sum_i A_ij (1 - A_ij) ||Q_i||_2,
 *   A = softmax(scale * Q K^T) with a causal mask, computed without materialising A
 *   from per-row statistics (row max, row sum) as in Alg. 1, and summed over the
 *   Hq/Hkv query heads that read a KV head.
 *
 *   q        fp16 [B][Hq][Nq][D]: the LAST Nq positions of an N-token context; query row i sits
 *            at position N-Nq+i and sees keys 0 .. N-Nq+i.  1 <= Nq <= N.
 *   k_fp16   fp16 [B][Hkv][N][D], the full-precision keys
 *   row_max, row_sum  optional fp32 [B][Hq][Nq] as an attention kernel extended per Sec. 3.3
 *            would supply them: row_max[i] = max_j scale*S_ij, row_sum[i] = sum_j exp(scale*S_ij - row_max[i]).
 *            Pass both or neither (NULL): with NULL the library computes them in a first pass.
 *   ans_k, ans_v      optional fp32 [B][Hkv][N] outputs (the scores); NULL = keep them in the workspace
 *   idx_k, idx_v      int32 [B][Hkv][k]: positions of the k highest AnS(K) / AnS(V) scores, ascending
 *            by position; equal scores resolve to the lower position.  0 <= k <= N.
 *            Either may be NULL to skip that selection.
 * Scores are accumulated in fp64 and rounded once to fp32; selection compares those fp32 values.
 */
size_t antkv_anchor_select_workspace(const antkv_geom* geom, int64_t N, int64_t Nq, int64_t k);
int antkv_anchor_select(const antkv_geom* geom, const void* q, const void* k_fp16, int64_t N,
                        int64_t Nq, float scale, int64_t k, const float* row_max,
                        const float* row_sum, float* ans_k, float* ans_v, int32_t* idx_k,
                        int32_t* idx_v, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Selection alone: for each of n_rows score rows (fp32 [n_rows][N], finite values), the positions
 * of the k largest, ascending; ties to the lower position.  idx: int32 [n_rows][k].
 */
size_t antkv_topk_workspace(int64_t n_rows, int64_t N, int64_t k);
int antkv_topk(const float* scores, int64_t n_rows, int64_t N, int64_t k, int32_t* idx,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Anchor store fill: rows_out[b][g][i][:] = x[b][g][idx[b][g][i]][:] (fp16 rows of D channels).
 *   x fp16 [B][Hkv][N][D]; idx int32 [B][Hkv][k] with entries in [0, N); rows_out fp16 [B][Hkv][k][D].
 */
int antkv_gather_rows(const antkv_geom* geom, const void* x, int64_t N, const int32_t* idx,
                      int64_t k, void* rows_out, void* stream);

/*
 * Decode attention for one new token per sequence (Attn of Sec. 2.1 with one query row):
 *   out[b][h] = softmax_j(scale * q[b][h] . K_eff[b][g][j]) . V_eff[b][g],   j = 0 .. N-1
 *   K_eff[j] = rows_k[slot] if j == idx_k[slot], else concat_m cb_k[g][m][codes_k[j][m]]
 *   V_eff[j] = rows_v[slot] if j == idx_v[slot], else concat_m cb_v[g][m][codes_v[j][m]]
 * (anchor tokens keep their FP16 rows, every other token is read from its codes; Fig. 2(b)).
 *
 *   q        fp16 [B][Hq][D]
 *   codes_k, codes_v  uint8 [B][Hkv][N_cap][code_bytes], tokens 0..N-1 valid (anchor positions hold codes
 *            too; they are ignored).  16-byte aligned.
 *   cb_k, cb_v        fp16 [Hkv][M][n_centroids][d_sub]
 *   idx_k    int32 [B][Hkv][k_k] strictly ascending in [0, N); rows_k fp16 [B][Hkv][k_k][D]
 *   idx_v, rows_v     likewise with k_v.  k_k and k_v may be 0 (pointers may then be NULL) up to N.
 *   out      fp16 [B][Hq][D]; accumulation is fp32, rounded once.
 * Precision: the scores of coded tokens are sums of fixed-point table entries q_h[m] . cb_k[g][m][c] with one quantum
 * per query head, R_h / 16256 for one-byte codes and R_h / 32767 for 12-bit codes, R_h being the largest
 * |scale * log2(e) * q_h[m] . cb_k[g][m][c]| over m and c.  The output stays within 2e-3 relative L2 of the exact
 * result while R_h <= L * 1e-3 / (ln 2 * sqrt(M / 12)) (L the number of levels above, M = D / d_sub sub-spaces:
 * about 14, 20, 29 for d_sub 4, 8, 16 and 82, 58 for the 12-bit formats with d_sub 32, 16); for larger entries the
 * bound grows in proportion to R_h (d_sub 8 and 16: unless ANTKV_DECODE_WIDE_TABLE is set, see
 * antkv_set_decode_options).  Anchor tokens are scored from their FP16 rows and are not affected.
 * Optional decode-time Anchor Score (Eq. (4) with the single query row over K_eff):
 *   ans_k, ans_v      fp32 [B][Hkv][N], both or neither (NULL):  ans_v[j] = sum_h p_hj,
 *            ans_k[j] = sum_h p_hj (1 - p_hj) ||q_h||_2
 *   resel_idx_k, resel_idx_v  int32 [B][Hkv][k_resel] or NULL: top-k_resel positions of those scores
 *            (ascending, ties to the lower position).  Needs ans_k / ans_v respectively to be non-NULL.
 * N == 0 writes zeros.  Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, ELAUNCH.
 */
size_t antkv_decode_attn_workspace(const antkv_geom* geom, int64_t N, int64_t k_k, int64_t k_v,
                                   int64_t k_resel);
int antkv_decode_attn(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                      const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k,
                      const void* cb_v, const int32_t* idx_k, const void* rows_k, int64_t k_k,
                      const int32_t* idx_v, const void* rows_v, int64_t k_v, void* out,
                      float* ans_k, float* ans_v, int32_t* resel_idx_k, int32_t* resel_idx_v,
                      int64_t k_resel, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Options of the one-byte-code decode kernel (antkv_decode_attn and the entry points built on it).  Process-wide mask;
 * takes effect for launches enqueued afterwards; returns the previous mask.  The default (0) is the fastest.
 *   ANTKV_DECODE_FIXED_ORDER  Reproducibility.  Codes, scores of antkv_anchor_select and index sets are the same on every
 *       run anyway.  The attention output is, by default, reproducible only to rounding level: after its first tile a wave
 *       pulls 64-token tiles from a counter, so the order of the fp32 sums varies from launch to launch.  With this bit
 *       every wave walks a fixed sequence of tiles: the output is then the same bit for bit for the same inputs, shape
 *       and workspace size, at a small cost in balance between the waves.  (The 12-bit kernels always work in a fixed
 *       order.)
 *   ANTKV_DECODE_WIDE_TABLE   Score range (see "Precision" at antkv_decode_attn).  The q . centroid table carries a
 *       second, residual entry per (code, sub-space): 30-bit instead of 15-bit fixed point, which lifts the limit on R_h
 *       for d_sub 8 and 16 at the price of a second table walk per token (about a quarter more time per step).
 *       d_sub 4 has no room for the second entry and ignores the bit; the 12-bit formats have 16-bit entries throughout.
 */
#define ANTKV_DECODE_FIXED_ORDER 1
#define ANTKV_DECODE_WIDE_TABLE 2
int antkv_set_decode_options(int options);

/*
 * Decode attention on a cache whose keys were stored BEFORE the rotary position embedding (Sec. 3.3, last paragraph:
 * the pre-RoPE strategy; Sec. 2.1 for RoPE on Q and K).  As antkv_decode_attn, with
 *   K_eff[j] = RoPE_{pos0 + j}( rows_k[slot] if j == idx_k[slot], else concat_m cb_k[g][m][codes_k[j][m]] ):
 * both the K codes and the FP16 K anchor rows hold un-rotated keys, and every key is rotated to its position when it
 * is used.  RoPE_p turns channel pair i = 0 .. D/2-1 by the angle p * rope_base^(-2 i / D); rope_style 0 pairs the
 * channels (2 i, 2 i + 1), rope_style 1 pairs (i, i + D/2).  q is used as given (the caller has rotated it to its own
 * position); values are untouched.  No Anchor Score outputs.
 * A first pass works out q_h . K_eff[j] for every token and head in fp32 (de-quantise, rotate, dot product; the rotated
 * keys are never written out) and leaves the scores in the workspace, 16 bytes per token and KV head; the decode kernels
 * then take their scores from there instead of from their lookup table, which has no meaning for keys that turn with
 * their position.  ANTKV_DECODE_FIXED_ORDER applies, ANTKV_DECODE_WIDE_TABLE does not (there is no table).
 * The workspace size comes from antkv_decode_attn_prerope_workspace(geom, N, k_v).
 * Errors: EINVAL (also rope_base <= 1, rope_style not 0 / 1, pos0 < 0), EUNSUPPORTED, EWORKSPACE, ELAUNCH.
 */
size_t antkv_decode_attn_prerope_workspace(const antkv_geom* geom, int64_t N, int64_t k_v);
int antkv_decode_attn_prerope(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                              const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k,
                              const void* cb_v, const int32_t* idx_k, const void* rows_k, int64_t k_k,
                              const int32_t* idx_v, const void* rows_v, int64_t k_v, float rope_base,
                              int rope_style, int64_t pos0, void* out, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * antkv_decode_attn for callers that cannot allocate device memory and therefore have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation and arguments as
 * antkv_decode_attn without the optional score / re-selection outputs and without the workspace: the kernels'
 * scratch (per-workgroup partial results and arrival words; for 12-bit codes also the K-side table) lives in an
 * array of ANTKV_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.
 * The call allocates nothing and frees nothing.  A shape whose scratch need
 * (antkv_decode_attn_workspace(geom, N, k_k, k_v, 0)) exceeds ANTKV_STATIC_SCRATCH_BYTES is refused with
 * ANTKV_EWORKSPACE before anything is enqueued.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (different streams, or this call next to another thread's) race and must be
 * serialised by the caller; nothing in the array has to be cleared between calls.
 */
#define ANTKV_STATIC_SCRATCH_BYTES (8u << 20)
int antkv_decode_attn_static(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                             const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k, const void* cb_v,
                             const int32_t* idx_k, const void* rows_k, int64_t k_k, const int32_t* idx_v,
                             const void* rows_v, int64_t k_v, void* out, void* stream);

/*
 * Decode append with an FP16 sliding window (Sec. 3.2, last paragraph: during decoding the Anchor Score's tail
 * locality is served by a sliding window of recent tokens kept in full precision; Sec. 4 uses a window of 32).
 * The window is the last W entries of BOTH anchor lists: before the call they are the positions N-W .. N-1.
 * The call (a) retires the oldest window token: its FP16 K / V rows are encoded against cb_k / cb_v (nearest centroid
 * per sub-vector with the lowest index among equal fp32 distances, as antkv_encode) into codes_k / codes_v at position N-W; (b) moves the other W-1 window entries one
 * place down; (c) stores k_new / v_new as the last entry with position N.  Afterwards the context has N+1 tokens
 * and the window is N-W+1 .. N; antkv_decode_attn can be called with N+1 and the same lists.  With W == 0 there is
 * no window: the new rows are encoded straight to position N.
 *
 *   k_new, v_new  fp16 [B][Hkv][D], 16-byte aligned
 *   codes_k, codes_v  uint8 [B][Hkv][N_cap][code_bytes];  N + 1 <= N_cap
 *   idx_k int32 [B][Hkv][k_k], rows_k fp16 [B][Hkv][k_k][D] (16-byte aligned), k_k >= W; likewise idx_v, rows_v, k_v.
 *   0 <= W <= 64, W <= N.
 * All work is enqueued on `stream` in order; nothing else may touch the lists or the codes meanwhile.
 * Errors: EINVAL, EUNSUPPORTED (W > 64), ELAUNCH.
 */
int antkv_append_token(const antkv_geom* geom, const void* k_new, const void* v_new, int64_t N, int64_t W,
                       const void* cb_k, const void* cb_v, uint8_t* codes_k, uint8_t* codes_v, int64_t N_cap,
                       int32_t* idx_k, void* rows_k, int64_t k_k, int32_t* idx_v, void* rows_v, int64_t k_v,
                       void* stream);

/*
 * Causal attention over the prompt (Sec. 2.1) that also returns the softmax row statistics, i.e. the
 * attention pass that Alg. 1 (Sec. 3.3) runs first and whose statistics antkv_anchor_select accepts.
 *
 *   q        fp16 [B][Hq][Nq][D]: the LAST Nq positions of an N-token context; query row i sits at
 *            position N-Nq+i and sees keys 0 .. N-Nq+i.  1 <= Nq <= N.
 *   k, v     fp16 [B][Hkv][N][D]; query head h reads KV head h / (Hq/Hkv)
 *   out      fp16 [B][Hq][Nq][D] = softmax(scale * q k^T, causal) v
 *   row_max, row_sum  optional fp32 [B][Hq][Nq] (both or neither): row_max[i] = max_j scale*S_ij,
 *            row_sum[i] = sum_j exp(scale*S_ij - row_max[i])
 * All pointers are device memory, 16-byte aligned; products are exact fp16 x fp16, accumulation is fp32,
 * probabilities enter the value product rounded to fp16.  No workspace.  geom.d_sub is not used but must
 * be valid.  Errors: EINVAL, ELAUNCH.
 */
int antkv_prefill_attn(const antkv_geom* geom, const void* q, const void* k, const void* v, int64_t N, int64_t Nq,
                       float scale, void* out, float* row_max, float* row_sum, void* stream);

/*
 * One iteration of the offline token-weighted k-means that learns a codebook (Sec. 3.1, "Offline Token-Aware
 * Centroids Learning"): every sub-vector of x is assigned to its nearest centroid of codebook_in (the same rule as
 * antkv_encode), then each centroid becomes the weighted mean of the sub-vectors assigned to it, over all B
 * sequences, with one weight per token (the paper uses the token's error-propagation factor; any w >= 0 works).
 * A centroid that no weight was assigned to keeps its old value.
 *
 *   x            fp16 [B][Hkv][n_tok][D] calibration rows of K (or V), contiguous, 16-byte aligned
 *   w            fp32 [B][Hkv][n_tok], >= 0
 *   codebook_in  fp16 [Hkv][M][n_centroids][d_sub];  codebook_out the same shape, a different buffer
 *   codes        uint8 [B][Hkv][n_tok][code_bytes], written: the assignment that was used
 *   wsum         optional fp32 [Hkv][M][n_centroids]: weight assigned to each centroid
 *   objective    optional fp64 [Hkv][M]: sum_j w_j ||x_j - codebook_in[code_j]||^2 per sub-space, i.e. the weighted
 *                distortion after the assignment and before the update
 *   workspace    antkv_kmeans_step_workspace(geom) bytes, 256-byte aligned; may hold any bytes on entry
 * Sums are fp32 and added with atomics: the new centroids agree to fp32 rounding from run to run, not bit for bit.
 * n_tok == 0 copies the codebook.  Errors: EINVAL, EUNSUPPORTED, EWORKSPACE, ELAUNCH.
 */
size_t antkv_kmeans_step_workspace(const antkv_geom* geom);
int antkv_kmeans_step(const antkv_geom* geom, const void* x, const float* w, int64_t n_tok, const void* codebook_in,
                      void* codebook_out, uint8_t* codes, float* wsum, double* objective, void* workspace,
                      size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ANTKV_H */
