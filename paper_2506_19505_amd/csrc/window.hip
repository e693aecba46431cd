// Decode append with an FP16 sliding window of recent tokens (paper Sec. 3.2, last paragraph; window of 32 in
// Sec. 4).  The window lives in the last W entries of the anchor lists.  One launch per step: a workgroup per
// (sequence, KV head, K|V) encodes the retiring token's row to its codes (nearest centroid per sub-vector,
// Sec. 3.1), moves the window one place down and appends the new token's row.  The step is latency-bound
// (one row per head), so the encode here is plain fp32 FMA work, one centroid per thread at a time, not the MFMA
// kernel.  With 4096 centroids (d_sub 32 or 16) a thread walks 16 of them per sub-space and the 12-bit codes are packed.
#include "common.h"

namespace antkv {

namespace {

constexpr int kApThreads = 256;   // thread c scores centroids c, c + 256, ... of every sub-space

// NC = centroids per sub-space: 256 (one code byte per sub-space) or 4096 (M 12-bit codes packed into 3 M / 2 bytes)
template <int DSUB, int NC>
__global__ __launch_bounds__(kApThreads) void append_kernel(
    const half_t* __restrict__ k_new, const half_t* __restrict__ v_new, const half_t* __restrict__ cb_k,
    const half_t* __restrict__ cb_v, uint8_t* __restrict__ codes_k, uint8_t* __restrict__ codes_v, int64_t N_cap,
    int32_t* __restrict__ idx_k, half_t* __restrict__ rows_k, int64_t k_k, int32_t* __restrict__ idx_v,
    half_t* __restrict__ rows_v, int64_t k_v, int64_t N, int W, int Hkv)
{
    constexpr int M = kD / DSUB;
    constexpr int kCodeBytes = NC == 256 ? M : 3 * M / 2;
    static_assert(NC == 256 || (NC == 4096 && M % 4 == 0), "12-bit codes are packed four to three 16-bit words");
    __shared__ float s_x[kD];
    __shared__ float s_val[M][4];
    __shared__ int s_idx[M][4];
    __shared__ int s_code[M];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bg = blockIdx.x;
    const int g = (int)(bg % Hkv);
    const bool is_v = blockIdx.y != 0;
    const int64_t kk = is_v ? k_v : k_k;
    half_t* rows = (is_v ? rows_v : rows_k) + (bg * kk + (kk - W)) * kD;          // first window row
    int32_t* idx = (is_v ? idx_v : idx_k) + bg * kk + (kk - W);
    const half_t* fresh = (is_v ? v_new : k_new) + bg * kD;
    const half_t* cb = (is_v ? cb_v : cb_k) + (size_t)g * kD * NC;
    uint8_t* codes = (is_v ? codes_v : codes_k) + (bg * N_cap + (N - W)) * kCodeBytes;   // codes of the retiring position

    // the row that becomes codes: the window's oldest, or the new row itself when there is no window
    const half_t* src = (W > 0) ? rows : fresh;
    if (tid < kD) s_x[tid] = (float)src[tid];
    // window moves are read now, written after the barrier below: up to 64 rows x 16 chunks, 4 per thread
    uint4_t mv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = tid + i * kApThreads, e = t >> 4, part = t & 15;
        mv[i] = uint4_t{0u, 0u, 0u, 0u};
        if (e < W) mv[i] = (e + 1 < W) ? ((const uint4_t*)rows)[(e + 1) * 16 + part] : ((const uint4_t*)fresh)[part];
    }
    __syncthreads();
    // thread t scores centroids t, t + 256, ... of every sub-space: x.c - |c|^2 / 2 (largest = nearest)
#pragma unroll 1
    for (int m = 0; m < M; ++m) {
        float val = -3.0e38f;
        int who = tid;
#pragma unroll 1
        for (int c = tid; c < NC; c += kApThreads) {                 // ascending, strict '>': ties keep the lower index
            const half_t* cen = cb + ((int64_t)m * NC + c) * DSUB;
            float cf[DSUB];
            if constexpr (DSUB == 4) {
                const half4_t v = *(const half4_t*)cen;
#pragma unroll
                for (int t = 0; t < 4; ++t) cf[t] = (float)v[t];
            } else {
#pragma unroll
                for (int u = 0; u < DSUB / 8; ++u) {
                    const half8_t v = *(const half8_t*)(cen + 8 * u);
#pragma unroll
                    for (int t = 0; t < 8; ++t) cf[8 * u + t] = (float)v[t];
                }
            }
            float nn = 0.f, dot = 0.f;
#pragma unroll
            for (int t = 0; t < DSUB; ++t) { nn = fmaf(cf[t], cf[t], nn); dot = fmaf(s_x[m * DSUB + t], cf[t], dot); }
            const float sc = fmaf(-0.5f, nn, dot);
            if (sc > val) { val = sc; who = c; }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {       // ties go to the lower centroid index
            const float ov = __shfl_xor(val, off, 64);
            const int oi = __shfl_xor(who, off, 64);
            if (ov > val || (ov == val && oi < who)) { val = ov; who = oi; }
        }
        if (lane == 0) { s_val[m][wave] = val; s_idx[m][wave] = who; }
    }
    __syncthreads();
    if (tid < M) {
        float val = s_val[tid][0];
        int who = s_idx[tid][0];
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (s_val[tid][w] > val || (s_val[tid][w] == val && s_idx[tid][w] < who)) { val = s_val[tid][w]; who = s_idx[tid][w]; }
        if constexpr (NC == 256) codes[tid] = (uint8_t)who;
        else s_code[tid] = who;
    }
    if constexpr (NC != 256) {                         // 12-bit codes, little-endian: code m at bits 12 m .. 12 m + 11
        __syncthreads();
        if (tid < M / 4) {
            const uint32_t c0 = (uint32_t)s_code[4 * tid], c1 = (uint32_t)s_code[4 * tid + 1];
            const uint32_t c2 = (uint32_t)s_code[4 * tid + 2], c3 = (uint32_t)s_code[4 * tid + 3];
            const uint32_t lo = c0 | (c1 << 12) | (c2 << 24);
            const uint32_t hi = (c2 >> 8) | (c3 << 4);
            uint16_t* dst = (uint16_t*)codes + 3 * tid;
            dst[0] = (uint16_t)lo;
            dst[1] = (uint16_t)(lo >> 16);
            dst[2] = (uint16_t)hi;
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = tid + i * kApThreads, e = t >> 4, part = t & 15;
        if (e < W) {
            ((uint4_t*)rows)[e * 16 + part] = mv[i];
            if (part == 0) idx[e] = (int32_t)(N - W + 1 + e);
        }
    }
}

}  // namespace

hipError_t launch_append(const Geom& g, const half_t* k_new, const half_t* v_new, const half_t* cb_k, const half_t* cb_v,
                         uint8_t* codes_k, uint8_t* codes_v, int64_t N_cap, int32_t* idx_k, half_t* rows_k, int64_t k_k,
                         int32_t* idx_v, half_t* rows_v, int64_t k_v, int64_t N, int W, hipStream_t st)
{
    if (g.B == 0) return hipSuccess;
    dim3 grid((unsigned)(g.B * g.Hkv), 2), block(kApThreads);
#define ANTKV_AP(DS, NCEN)                                                                                           \
    hipLaunchKernelGGL((append_kernel<DS, NCEN>), grid, block, 0, st, k_new, v_new, cb_k, cb_v, codes_k, codes_v, N_cap, \
                       idx_k, rows_k, k_k, idx_v, rows_v, k_v, N, W, g.Hkv)
    if (g.C == 4096 && g.d == 32) ANTKV_AP(32, 4096);
    else if (g.C == 4096) ANTKV_AP(16, 4096);
    else if (g.d == 4) ANTKV_AP(4, 256);
    else if (g.d == 8) ANTKV_AP(8, 256);
    else ANTKV_AP(16, 256);
#undef ANTKV_AP
    return hipGetLastError();
}

}  // namespace antkv
