// Shared declarations of the AnTKV HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/antkv.h"

namespace antkv {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half16_t __attribute__((ext_vector_type(16)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef int int4_t __attribute__((ext_vector_type(4)));

constexpr int kD = 128;          // head dim
constexpr int kC = 256;          // centroids per sub-space
constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;   // stands for -inf in running maxima (exp2 of it is 0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- device helpers -------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Wait until every global load issued so far has landed.  Placed after the loads of a loop-invariant register
// tile: the compiler otherwise keeps those loads "possibly pending" across the loop's back edge and makes the
// loop body wait for its own prefetches of the next tile before it may touch the invariant registers.
// (pin() on the loaded registers first keeps the compiler from moving their loads below the wait)
template <typename T>
__device__ __forceinline__ void pin(T& x)
{
    asm volatile("" : "+v"(x));
}
__device__ __forceinline__ void wait_all_loads()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
    asm volatile("" ::: "memory");
}

// order-preserving map float -> uint32 (larger float <=> larger key), any finite sign
__device__ __forceinline__ uint32_t float_key(float f)
{
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// ---- launchers (each enqueues on `stream` and returns a hipError_t) --------------------------
struct Geom {
    int B, Hq, Hkv, G, d, M;
    int C;            // centroids per sub-space: 256 (one byte per code) or 4096 (12-bit codes, d = 32 or 16)
    int code_bytes;   // bytes of one token's codes: M, or 3 M / 2 for packed 12-bit codes (6 for d = 32, 12 for d = 16)
};

hipError_t launch_encode(const Geom& g, const half_t* x, int64_t xs_b, int64_t xs_h, int64_t xs_t,
                         int64_t n_tok, const half_t* cb, uint8_t* codes, int64_t N_cap,
                         int64_t token_offset, hipStream_t st);

hipError_t launch_encode12(const Geom& g, const half_t* x, int64_t xs_b, int64_t xs_h, int64_t xs_t,
                           int64_t n_tok, const half_t* cb, uint8_t* codes, int64_t N_cap,
                           int64_t token_offset, hipStream_t st);

size_t topk_workspace_bytes(int64_t n_rows, int64_t N, int64_t k);
hipError_t launch_topk(const float* scores, int64_t n_rows, int64_t N, int64_t k, int32_t* idx,
                       void* ws, hipStream_t st);
hipError_t launch_topk2(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                        int64_t N, int64_t k, void* ws, hipStream_t st);
// The same selection in two halves, for a producer that counts its scores while it writes them: `begin` clears the
// workspace's counters and returns the first-level histograms, uint32 [2 n_rows][2 * kTopkBins] (row r < n_rows belongs
// to scores row r, row n_rows + r to scores_b row r; the first kTopkBins words of a row count float_key(score) >> 21);
// the producer adds every score it writes to them; `finish` selects from there without reading the scores for a histogram.
constexpr int kTopkBins = 2048;
uint32_t* launch_topk2_begin(int64_t n_rows, int64_t N, void* ws, hipStream_t st);
hipError_t launch_topk2_finish(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                               int64_t N, int64_t k, void* ws, hipStream_t st);

hipError_t launch_gather_rows(const Geom& g, const half_t* x, int64_t N, const int32_t* idx,
                              int64_t k, half_t* rows, hipStream_t st);
hipError_t launch_append(const Geom& g, const half_t* k_new, const half_t* v_new, const half_t* cb_k, const half_t* cb_v,
                         uint8_t* codes_k, uint8_t* codes_v, int64_t N_cap, int32_t* idx_k, half_t* rows_k, int64_t k_k,
                         int32_t* idx_v, half_t* rows_v, int64_t k_v, int64_t N, int W, hipStream_t st);

size_t anchor_score_workspace_bytes(const Geom& g, int64_t N, int64_t Nq);
size_t kmeans_workspace_bytes(const Geom& g);
hipError_t launch_kmeans_update(const Geom& g, const half_t* x, const float* w, int64_t n_tok, const half_t* cb_in,
                                half_t* cb_out, const uint8_t* codes, float* wsum_out, double* objective, void* ws,
                                hipStream_t st);
hipError_t launch_prefill_attn(const Geom& g, const half_t* q, const half_t* k, const half_t* v, int64_t N, int64_t Nq,
                               float scale, half_t* out, float* row_max, float* row_sum, hipStream_t st);
hipError_t launch_anchor_score(const Geom& g, const half_t* q, const half_t* k, int64_t N, int64_t Nq,
                               float scale, const float* row_max, const float* row_sum,
                               float* ans_k, float* ans_v, void* ws, hipStream_t st);

struct DecodeArgs {
    const half_t* q;
    float scale;
    const uint8_t *codes_k, *codes_v;
    int64_t N, N_cap;
    const half_t *cb_k, *cb_v;
    const int32_t* idx_k;
    const half_t* rows_k;
    int64_t k_k;
    const int32_t* idx_v;
    const half_t* rows_v;
    int64_t k_v;
    half_t* out;
    float *ans_k, *ans_v;
    uint32_t* topk_hist;   // optional: first-level top-k histograms that the score pass fills (see launch_topk2_begin)
    // optional (k_k = 0, no Anchor Scores): the K side's scores in log2 units as launch_rope_scores writes them (one-byte
    // codes: grouped by four tokens; 12-bit codes: [B][Hkv][N][4 heads]); the K codes, the K codebook and scale are then not used
    const float* given_scores = nullptr;
};
int set_decode_options(int options);   // ANTKV_DECODE_* mask; returns the previous mask
int decode_num_splits(const Geom& g, int64_t N);
size_t decode_workspace_bytes(const Geom& g, int64_t N, int64_t k_k, int64_t k_v, bool want_ans);
hipError_t launch_decode_attn(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st);
// scores_out fp32 = scale * log2(e) * q_h . RoPE_{pos0 + j}(K_eff[j]) for the group's heads (K_eff: the FP16 anchor row or the
// centroids of the codes), in the layout that DecodeArgs::given_scores describes
hipError_t launch_rope_scores(const Geom& g, const half_t* q, float scale, const uint8_t* codes_k, int64_t N, int64_t N_cap,
                              const half_t* cb_k, const int32_t* idx_k, const half_t* rows_k, int64_t k_k, double rope_base,
                              int rope_style, int64_t pos0, float* scores_out, hipStream_t st);
size_t decode12_workspace_bytes(const Geom& g, int64_t N);
hipError_t launch_decode12(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st);

}  // namespace antkv
