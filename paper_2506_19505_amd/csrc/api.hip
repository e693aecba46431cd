// extern "C" boundary of the AnTKV library: argument validation, workspace layout, kernel launches.
#include "common.h"

#include <mutex>

using namespace antkv;

namespace {

int check_geom(const antkv_geom* gm, Geom& g)
{
    if (!gm) return ANTKV_EINVAL;
    if (gm->B < 0 || gm->Hq <= 0 || gm->Hkv <= 0 || gm->D <= 0 || gm->d_sub <= 0 || gm->n_centroids <= 0)
        return ANTKV_EINVAL;
    if (gm->Hq % gm->Hkv != 0) return ANTKV_EINVAL;
    if (gm->D != kD) return ANTKV_EUNSUPPORTED;
    const bool wide = gm->n_centroids == 4096 && (gm->d_sub == 32 || gm->d_sub == 16);   // 12-bit codes
    const bool byte_codes = gm->n_centroids == kC && (gm->d_sub == 4 || gm->d_sub == 8 || gm->d_sub == 16);
    if (!wide && !byte_codes) return ANTKV_EUNSUPPORTED;
    const int G = gm->Hq / gm->Hkv;
    if (G != 1 && G != 2 && G != 4) return ANTKV_EUNSUPPORTED;
    if ((int64_t)gm->B * gm->Hkv > 65535) return ANTKV_EUNSUPPORTED;
    g.B = gm->B; g.Hq = gm->Hq; g.Hkv = gm->Hkv; g.G = G; g.d = gm->d_sub; g.M = kD / gm->d_sub;
    g.C = gm->n_centroids;
    g.code_bytes = wide ? 3 * g.M / 2 : g.M;
    return ANTKV_OK;
}

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

struct SelPlan {
    size_t off_score, off_topk, total;
};

SelPlan sel_plan(const Geom& g, int64_t N, int64_t Nq, int64_t k)
{
    SelPlan p;
    p.off_score = 0;
    p.off_topk = align_up(anchor_score_workspace_bytes(g, N, Nq));
    p.total = p.off_topk + align_up(topk_workspace_bytes(2 * (int64_t)g.B * g.Hkv, N, k));   // K and V rows in one go
    return p;
}

struct DecPlan {
    size_t off_dec, off_topk, total;
};

DecPlan dec_plan(const Geom& g, int64_t N, int64_t k_k, int64_t k_v, int64_t k_resel, bool want_ans)
{
    DecPlan p;
    p.off_dec = 0;
    p.off_topk = align_up(decode_workspace_bytes(g, N, k_k, k_v, want_ans));
    p.total = p.off_topk + (k_resel > 0 ? align_up(topk_workspace_bytes(2 * (int64_t)g.B * g.Hkv, N, k_resel)) : 0);
    return p;
}

int decode_attn_impl(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                      const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k, const void* cb_v,
                      const int32_t* idx_k, const void* rows_k, int64_t k_k, const int32_t* idx_v, const void* rows_v,
                      int64_t k_v, void* out, float* ans_k, float* ans_v, int32_t* resel_idx_k, int32_t* resel_idx_v,
                      int64_t k_resel, void* workspace, size_t workspace_bytes, void* stream,
                      const float* given_scores = nullptr)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N < 0 || N_cap < N || k_k < 0 || k_v < 0 || k_k > N || k_v > N || k_resel < 0 || k_resel > N ||
        N > 0x7fffffffLL)
        return ANTKV_EINVAL;
    const bool wide = g.C != kC;                                 // 12-bit codes
    if (g.B == 0) return ANTKV_OK;
    if (!q || !out || misaligned(q, 16) || misaligned(out, 16)) return ANTKV_EINVAL;
    if (!(scale > 0.f)) return ANTKV_EINVAL;
    if (N > 0) {
        if (!codes_k || !codes_v || !cb_k || !cb_v) return ANTKV_EINVAL;
        if (misaligned(codes_k, 16) || misaligned(codes_v, 16) || misaligned(cb_k, 16) || misaligned(cb_v, 16))
            return ANTKV_EINVAL;
        if (k_k > 0 && (!idx_k || !rows_k || misaligned(rows_k, 16))) return ANTKV_EINVAL;
        if (k_v > 0 && (!idx_v || !rows_v || misaligned(rows_v, 16))) return ANTKV_EINVAL;
    }
    if ((resel_idx_k && !ans_k) || (resel_idx_v && !ans_v)) return ANTKV_EINVAL;
    const bool want_ans = ans_k || ans_v;
    if (want_ans && !(ans_k && ans_v)) return ANTKV_EINVAL;   // the two scores are produced together
    if (wide) {
        const size_t off_topk = align_up(decode12_workspace_bytes(g, N));
        const size_t need = off_topk + (k_resel > 0 ? align_up(topk_workspace_bytes(2 * (int64_t)g.B * g.Hkv, N, k_resel)) : 0);
        if (!workspace || misaligned(workspace, 256) || workspace_bytes < need) return ANTKV_EWORKSPACE;
        hipStream_t st = (hipStream_t)stream;
        DecodeArgs a;
        a.q = (const half_t*)q; a.scale = scale; a.codes_k = codes_k; a.codes_v = codes_v; a.N = N; a.N_cap = N_cap;
        a.cb_k = (const half_t*)cb_k; a.cb_v = (const half_t*)cb_v; a.idx_k = idx_k; a.rows_k = (const half_t*)rows_k;
        a.k_k = k_k; a.idx_v = idx_v; a.rows_v = (const half_t*)rows_v; a.k_v = k_v; a.out = (half_t*)out;
        a.ans_k = ans_k; a.ans_v = ans_v;
        a.given_scores = given_scores;
        // with both index sets wanted, the score pass counts its scores into the selection's first histogram
        const bool fused = N > 0 && k_resel > 0 && resel_idx_k && resel_idx_v;
        a.topk_hist = fused ? launch_topk2_begin((int64_t)g.B * g.Hkv, N, (char*)workspace + off_topk, st) : nullptr;
        if (launch_decode12(g, a, workspace, st) != hipSuccess) return ANTKV_ELAUNCH;
        if (N > 0 && k_resel > 0 && (resel_idx_k || resel_idx_v)) {
            char* w = (char*)workspace;
            const int64_t rows = (int64_t)g.B * g.Hkv;
            const hipError_t e =
                (resel_idx_k && resel_idx_v)
                    ? launch_topk2_finish(ans_k, resel_idx_k, ans_v, resel_idx_v, rows, N, k_resel, w + off_topk, st)
                    : launch_topk(resel_idx_k ? ans_k : ans_v, rows, N, k_resel, resel_idx_k ? resel_idx_k : resel_idx_v,
                                  w + off_topk, st);
            if (e != hipSuccess) return ANTKV_ELAUNCH;
        }
        return ANTKV_OK;
    }
    const DecPlan dp = dec_plan(g, N, k_k, k_v, k_resel, true);
    if (N > 0 && (!workspace || misaligned(workspace, 256) || workspace_bytes < dp.total)) return ANTKV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    DecodeArgs a;
    a.q = (const half_t*)q; a.scale = scale; a.codes_k = codes_k; a.codes_v = codes_v; a.N = N; a.N_cap = N_cap;
    a.cb_k = (const half_t*)cb_k; a.cb_v = (const half_t*)cb_v; a.idx_k = idx_k; a.rows_k = (const half_t*)rows_k;
    a.k_k = k_k; a.idx_v = idx_v; a.rows_v = (const half_t*)rows_v; a.k_v = k_v; a.out = (half_t*)out;
    a.ans_k = ans_k; a.ans_v = ans_v;
    a.given_scores = given_scores;
    // with both index sets wanted, the score pass counts its scores into the selection's first histogram
    const bool fused = N > 0 && k_resel > 0 && resel_idx_k && resel_idx_v;
    a.topk_hist = fused ? launch_topk2_begin((int64_t)g.B * g.Hkv, N, (char*)workspace + dp.off_topk, st) : nullptr;
    hipError_t e = launch_decode_attn(g, a, workspace, st);
    if (e != hipSuccess) return ANTKV_ELAUNCH;
    if (N > 0 && k_resel > 0) {
        char* w = (char*)workspace;
        const int64_t rows = (int64_t)g.B * g.Hkv;
        if (resel_idx_k && resel_idx_v) {
            e = launch_topk2_finish(ans_k, resel_idx_k, ans_v, resel_idx_v, rows, N, k_resel, w + dp.off_topk, st);
            if (e != hipSuccess) return ANTKV_ELAUNCH;
        } else if (resel_idx_k || resel_idx_v) {
            e = launch_topk(resel_idx_k ? ans_k : ans_v, rows, N, k_resel, resel_idx_k ? resel_idx_k : resel_idx_v,
                            w + dp.off_topk, st);
            if (e != hipSuccess) return ANTKV_ELAUNCH;
        }
    }
    return ANTKV_OK;
}


// ---- scratch of the entry point that takes no workspace --------------------------------------------------------
// One array per GPU, held from the moment the library is loaded on it until the process ends.  Host code never
// uses the array's name as an address: the device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[ANTKV_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ANTKV_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ANTKV_ELAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return ANTKV_OK;
}

}  // namespace

extern "C" {

int antkv_version(void) { return 1; }

const char* antkv_strerror(int code)
{
    switch (code) {
    case ANTKV_OK: return "ok";
    case ANTKV_EINVAL: return "invalid argument";
    case ANTKV_EUNSUPPORTED: return "unsupported geometry";
    case ANTKV_EWORKSPACE: return "workspace missing or too small";
    case ANTKV_ELAUNCH: return "HIP launch failed";
    default: return "unknown error";
    }
}

int antkv_encode(const antkv_geom* geom, const void* x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
                 const void* codebook, uint8_t* codes, int64_t N_cap, int64_t token_offset, void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (n_tok < 0 || N_cap < 0 || token_offset < 0 || token_offset + n_tok > N_cap) return ANTKV_EINVAL;
    if (n_tok == 0 || g.B == 0) return ANTKV_OK;
    if (!x || !codebook || !codes) return ANTKV_EINVAL;
    if (misaligned(x, 16) || misaligned(codebook, 16) || misaligned(codes, 16)) return ANTKV_EINVAL;
    if (xs_t < kD || (xs_b & 7) || (xs_h & 7) || (xs_t & 7) || xs_b < 0 || xs_h < 0) return ANTKV_EINVAL;
    const hipError_t e =
        g.C == 4096 ? launch_encode12(g, (const half_t*)x, xs_b, xs_h, xs_t, n_tok, (const half_t*)codebook, codes, N_cap,
                                      token_offset, (hipStream_t)stream)
                    : launch_encode(g, (const half_t*)x, xs_b, xs_h, xs_t, n_tok, (const half_t*)codebook, codes, N_cap,
                                    token_offset, (hipStream_t)stream);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

size_t antkv_topk_workspace(int64_t n_rows, int64_t N, int64_t k)
{
    if (n_rows < 0 || N < 0 || k < 0) return 0;
    return topk_workspace_bytes(n_rows, N, k);
}

int antkv_topk(const float* scores, int64_t n_rows, int64_t N, int64_t k, int32_t* idx, void* workspace,
               size_t workspace_bytes, void* stream)
{
    if (n_rows < 0 || N < 0 || k < 0 || k > N || N > 0x7fffffffLL || n_rows > 65535) return ANTKV_EINVAL;
    if (k == 0 || n_rows == 0) return ANTKV_OK;
    if (!scores || !idx) return ANTKV_EINVAL;
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < topk_workspace_bytes(n_rows, N, k))
        return ANTKV_EWORKSPACE;
    hipError_t e = launch_topk(scores, n_rows, N, k, idx, workspace, (hipStream_t)stream);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

size_t antkv_anchor_select_workspace(const antkv_geom* geom, int64_t N, int64_t Nq, int64_t k)
{
    Geom g;
    if (check_geom(geom, g) || N <= 0 || Nq <= 0 || Nq > N || k < 0) return 0;
    return sel_plan(g, N, Nq, k).total;
}

size_t antkv_kmeans_step_workspace(const antkv_geom* geom)
{
    Geom g;
    if (check_geom(geom, g)) return 0;
    return kmeans_workspace_bytes(g);
}

int antkv_kmeans_step(const antkv_geom* geom, const void* x, const float* w, int64_t n_tok, const void* codebook_in,
                      void* codebook_out, uint8_t* codes, float* wsum, double* objective, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (n_tok < 0 || n_tok > 0x7fffffffLL) return ANTKV_EINVAL;
    if (!codebook_in || !codebook_out || codebook_in == codebook_out) return ANTKV_EINVAL;
    if (misaligned(codebook_in, 16) || misaligned(codebook_out, 16) || misaligned(objective, 8)) return ANTKV_EINVAL;
    const bool have_tokens = n_tok > 0 && g.B > 0;
    if (have_tokens && (!x || !w || !codes || misaligned(x, 16) || misaligned(codes, 16) || misaligned(w, 4)))
        return ANTKV_EINVAL;
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < kmeans_workspace_bytes(g)) return ANTKV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (have_tokens) {
        const hipError_t e =
            g.C == kC ? launch_encode(g, (const half_t*)x, (int64_t)g.Hkv * n_tok * kD, n_tok * kD, kD, n_tok,
                                      (const half_t*)codebook_in, codes, n_tok, 0, st)
                      : launch_encode12(g, (const half_t*)x, (int64_t)g.Hkv * n_tok * kD, n_tok * kD, kD, n_tok,
                                        (const half_t*)codebook_in, codes, n_tok, 0, st);
        if (e != hipSuccess) return ANTKV_ELAUNCH;
    }
    const hipError_t e = launch_kmeans_update(g, (const half_t*)x, w, have_tokens ? n_tok : 0, (const half_t*)codebook_in,
                                              (half_t*)codebook_out, codes, wsum, objective, workspace, st);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

int antkv_prefill_attn(const antkv_geom* geom, const void* q, const void* k, const void* v, int64_t N, int64_t Nq,
                       float scale, void* out, float* row_max, float* row_sum, void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N <= 0 || Nq <= 0 || Nq > N || N > 0x7fffffffLL) return ANTKV_EINVAL;
    if ((row_max == nullptr) != (row_sum == nullptr)) return ANTKV_EINVAL;
    if (g.B == 0) return ANTKV_OK;
    if (!q || !k || !v || !out) return ANTKV_EINVAL;
    if (misaligned(q, 16) || misaligned(k, 16) || misaligned(v, 16) || misaligned(out, 16)) return ANTKV_EINVAL;
    if (!(scale > 0.f)) return ANTKV_EINVAL;
    const hipError_t e = launch_prefill_attn(g, (const half_t*)q, (const half_t*)k, (const half_t*)v, N, Nq, scale,
                                             (half_t*)out, row_max, row_sum, (hipStream_t)stream);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

int antkv_anchor_select(const antkv_geom* geom, const void* q, const void* k_fp16, int64_t N, int64_t Nq, float scale,
                        int64_t k, const float* row_max, const float* row_sum, float* ans_k, float* ans_v,
                        int32_t* idx_k, int32_t* idx_v, void* workspace, size_t workspace_bytes, void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N <= 0 || Nq <= 0 || Nq > N || k < 0 || k > N || N > 0x7fffffffLL) return ANTKV_EINVAL;
    if ((row_max == nullptr) != (row_sum == nullptr)) return ANTKV_EINVAL;
    if (g.B == 0) return ANTKV_OK;
    if (!q || !k_fp16) return ANTKV_EINVAL;
    if (misaligned(q, 16) || misaligned(k_fp16, 16)) return ANTKV_EINVAL;
    if (!(scale > 0.f)) return ANTKV_EINVAL;
    const SelPlan sp = sel_plan(g, N, Nq, k);
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < sp.total) return ANTKV_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)workspace;
    // scores default to the tail of the score workspace
    const size_t as_bytes = anchor_score_workspace_bytes(g, N, Nq);
    const size_t score_bytes = align_up((size_t)g.B * g.Hkv * N * sizeof(float));
    float* sk = ans_k ? ans_k : (float*)(w + as_bytes - 2 * score_bytes);
    float* sv = ans_v ? ans_v : (float*)(w + as_bytes - score_bytes);
    hipError_t e = launch_anchor_score(g, (const half_t*)q, (const half_t*)k_fp16, N, Nq, scale, row_max, row_sum, sk, sv,
                                       w + sp.off_score, st);
    if (e != hipSuccess) return ANTKV_ELAUNCH;
    const int64_t rows = (int64_t)g.B * g.Hkv;
    if (idx_k && idx_v && k > 0) {
        e = launch_topk2(sk, idx_k, sv, idx_v, rows, N, k, w + sp.off_topk, st);
        if (e != hipSuccess) return ANTKV_ELAUNCH;
    } else if ((idx_k || idx_v) && k > 0) {
        e = launch_topk(idx_k ? sk : sv, rows, N, k, idx_k ? idx_k : idx_v, w + sp.off_topk, st);
        if (e != hipSuccess) return ANTKV_ELAUNCH;
    }
    return ANTKV_OK;
}

int antkv_gather_rows(const antkv_geom* geom, const void* x, int64_t N, const int32_t* idx, int64_t k, void* rows_out,
                      void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N < 0 || k < 0 || k > N) return ANTKV_EINVAL;
    if (k == 0 || g.B == 0) return ANTKV_OK;
    if (!x || !idx || !rows_out || misaligned(x, 16) || misaligned(rows_out, 16)) return ANTKV_EINVAL;
    hipError_t e = launch_gather_rows(g, (const half_t*)x, N, idx, k, (half_t*)rows_out, (hipStream_t)stream);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

int antkv_append_token(const antkv_geom* geom, const void* k_new, const void* v_new, int64_t N, int64_t W,
                       const void* cb_k, const void* cb_v, uint8_t* codes_k, uint8_t* codes_v, int64_t N_cap,
                       int32_t* idx_k, void* rows_k, int64_t k_k, int32_t* idx_v, void* rows_v, int64_t k_v,
                       void* stream)
{
    Geom g;
    int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N < 0 || W < 0 || W > N || N + 1 > N_cap || k_k < W || k_v < W) return ANTKV_EINVAL;
    if (W > 64) return ANTKV_EUNSUPPORTED;
    if (g.B == 0) return ANTKV_OK;
    if (!k_new || !v_new || !cb_k || !cb_v || !codes_k || !codes_v || misaligned(k_new, 16) || misaligned(v_new, 16) ||
        misaligned(cb_k, 16) || misaligned(cb_v, 16) || misaligned(codes_k, 16) || misaligned(codes_v, 16))
        return ANTKV_EINVAL;
    if (W > 0 && (!idx_k || !rows_k || !idx_v || !rows_v || misaligned(rows_k, 16) || misaligned(rows_v, 16)))
        return ANTKV_EINVAL;
    hipError_t e = launch_append(g, (const half_t*)k_new, (const half_t*)v_new, (const half_t*)cb_k, (const half_t*)cb_v,
                                 codes_k, codes_v, N_cap, idx_k, (half_t*)rows_k, k_k, idx_v, (half_t*)rows_v, k_v, N, (int)W,
                                 (hipStream_t)stream);
    return e == hipSuccess ? ANTKV_OK : ANTKV_ELAUNCH;
}

size_t antkv_decode_attn_workspace(const antkv_geom* geom, int64_t N, int64_t k_k, int64_t k_v, int64_t k_resel)
{
    Geom g;
    if (check_geom(geom, g) || N < 0 || k_k < 0 || k_v < 0 || k_resel < 0) return 0;
    if (g.C != kC)
        return align_up(decode12_workspace_bytes(g, N)) +
               (k_resel > 0 ? align_up(topk_workspace_bytes(2 * (int64_t)g.B * g.Hkv, N, k_resel)) : 0);
    return dec_plan(g, N, k_k, k_v, k_resel, true).total;
}

int antkv_decode_attn(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                      const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k, const void* cb_v,
                      const int32_t* idx_k, const void* rows_k, int64_t k_k, const int32_t* idx_v, const void* rows_v,
                      int64_t k_v, void* out, float* ans_k, float* ans_v, int32_t* resel_idx_k, int32_t* resel_idx_v,
                      int64_t k_resel, void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_attn_impl(geom, q, scale, codes_k, codes_v, N, N_cap, cb_k, cb_v, idx_k, rows_k, k_k, idx_v, rows_v, k_v,
                            out, ans_k, ans_v, resel_idx_k, resel_idx_v, k_resel, workspace, workspace_bytes, stream);
}

int antkv_set_decode_options(int options) { return set_decode_options(options); }

// bytes of the K side's scores that the pre-RoPE path keeps in its workspace: 16 per token and KV head (one-byte codes:
// tokens rounded up to 64, the decode kernel reads whole tiles)
static size_t prerope_score_bytes(const Geom& g, int64_t N)
{
    const int64_t n = g.C == kC ? (N + 63) / 64 * 64 : N;
    return align_up((size_t)g.B * g.Hkv * (size_t)n * 16);
}

size_t antkv_decode_attn_prerope_workspace(const antkv_geom* geom, int64_t N, int64_t k_v)
{
    Geom g;
    if (check_geom(geom, g) || N < 0 || k_v < 0) return 0;
    return prerope_score_bytes(g, N) + align_up(antkv_decode_attn_workspace(geom, N, 0, k_v, 0));
}

int antkv_decode_attn_prerope(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                              const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k, const void* cb_v,
                              const int32_t* idx_k, const void* rows_k, int64_t k_k, const int32_t* idx_v,
                              const void* rows_v, int64_t k_v, float rope_base, int rope_style, int64_t pos0, void* out,
                              void* workspace, size_t workspace_bytes, void* stream)
{
    Geom g;
    const int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N < 0 || N_cap < N || k_k < 0 || k_v < 0 || k_k > N || k_v > N || N > 0x7fffffffLL) return ANTKV_EINVAL;
    if (!(rope_base > 1.f) || (rope_style != 0 && rope_style != 1) || pos0 < 0 || pos0 > (1LL << 40)) return ANTKV_EINVAL;
    if (g.B == 0) return ANTKV_OK;
    if (N == 0)   // nothing to rotate: the plain call writes the zeros
        return decode_attn_impl(geom, q, scale, codes_k, codes_v, 0, N_cap, cb_k, cb_v, nullptr, nullptr, 0, nullptr, nullptr, 0,
                                out, nullptr, nullptr, nullptr, nullptr, 0, workspace, workspace_bytes, stream);
    if (!codes_k || !cb_k || misaligned(codes_k, 16) || misaligned(cb_k, 16)) return ANTKV_EINVAL;
    if (k_k > 0 && (!idx_k || !rows_k || misaligned(rows_k, 16))) return ANTKV_EINVAL;
    if (!q || misaligned(q, 16) || !(scale > 0.f)) return ANTKV_EINVAL;
    const size_t need = antkv_decode_attn_prerope_workspace(geom, N, k_v);
    if (!workspace || misaligned(workspace, 256) || workspace_bytes < need) return ANTKV_EWORKSPACE;
    // The rotated keys are never written out: a first pass leaves q . RoPE(K_eff) of every token and head (FP16 anchor
    // rows included) in the workspace, and the decode kernels take their scores from there instead of from a table.
    char* w = (char*)workspace;
    const size_t sc_b = prerope_score_bytes(g, N);
    if (launch_rope_scores(g, (const half_t*)q, scale, codes_k, N, N_cap, (const half_t*)cb_k, idx_k, (const half_t*)rows_k, k_k,
                           (double)rope_base, rope_style, pos0, (float*)w, (hipStream_t)stream) != hipSuccess)
        return ANTKV_ELAUNCH;
    return decode_attn_impl(geom, q, scale, codes_k, codes_v, N, N_cap, cb_k, cb_v, nullptr, nullptr, 0, idx_v, rows_v, k_v, out,
                            nullptr, nullptr, nullptr, nullptr, 0, w + sc_b, workspace_bytes - sc_b, stream, (const float*)w);
}

int antkv_decode_attn_static(const antkv_geom* geom, const void* q, float scale, const uint8_t* codes_k,
                             const uint8_t* codes_v, int64_t N, int64_t N_cap, const void* cb_k, const void* cb_v,
                             const int32_t* idx_k, const void* rows_k, int64_t k_k, const int32_t* idx_v,
                             const void* rows_v, int64_t k_v, void* out, void* stream)
{
    Geom g;
    const int rc = check_geom(geom, g);
    if (rc) return rc;
    if (N < 0 || k_k < 0 || k_v < 0) return ANTKV_EINVAL;
    const size_t need = antkv_decode_attn_workspace(geom, N, k_k, k_v, 0);
    if (need > (size_t)ANTKV_STATIC_SCRATCH_BYTES) return ANTKV_EWORKSPACE;   // shape beyond the built-in scratch
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs) return rs;
    return decode_attn_impl(geom, q, scale, codes_k, codes_v, N, N_cap, cb_k, cb_v, idx_k, rows_k, k_k, idx_v, rows_v, k_v,
                            out, nullptr, nullptr, nullptr, nullptr, 0, ws, (size_t)ANTKV_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"
