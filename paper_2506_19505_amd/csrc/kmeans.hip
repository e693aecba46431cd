// One iteration of the offline token-weighted k-means that learns the codebooks (paper Sec. 3.1, "Offline
// Token-Aware Centroids Learning": the sub-vectors of K / V are clustered with one weight per token, the weight
// standing for that token's error-propagation factor).  The assignment step is the online encode kernel; this file
// holds the update step: per (KV head, sub-space, centroid) the weighted sum of the assigned sub-vectors and the
// assigned weight, then the weighted mean.
//
// Accumulation: a workgroup takes a chunk of tokens and a quarter of the sub-spaces, adds w*x and w into fp32
// accumulators in LDS (ds_add_f32; laid out [sub-space][channel][centroid] so that the lanes of one instruction
// spread over the banks by their codes), and flushes the non-zero accumulators to the global sums with hardware float atomics.  Sums are
// therefore fp32 and their order is not fixed: results agree to fp32 rounding, not bit for bit, from run to run.
// With 4096 centroids (12-bit codes) the sums of one KV head are 2 MB, far beyond LDS, and 4096 targets per sub-space
// rarely collide, so every thread adds its eight channels straight into the global sums (km_accumulate12).
#include "common.h"

namespace antkv {

namespace {

constexpr int kKmThreads = 256;
constexpr int kKmChunk = 2048;     // tokens per workgroup
constexpr int kKmGroups = 4;       // sub-space groups (grid.z)

__global__ __launch_bounds__(256) void km_zero(uint32_t* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

template <int DSUB>
__global__ __launch_bounds__(kKmThreads) void km_accumulate(
    const half_t* __restrict__ x, const float* __restrict__ w, const uint8_t* __restrict__ codes,
    const half_t* __restrict__ cb, int64_t n_tok, int Hkv, float* __restrict__ sums, float* __restrict__ wsum,
    double* __restrict__ objective)
{
    constexpr int M = kD / DSUB, MG = M / kKmGroups;            // sub-spaces per workgroup: 8 / 4 / 2
    __shared__ float s_sum[MG * kC * DSUB];                     // 32 KB
    __shared__ float s_w[MG * kC];
    const int tid = threadIdx.x;
    const int64_t bg = blockIdx.y;
    const int g = (int)(bg % Hkv);
    const int m0 = blockIdx.z * MG;
    for (int i = tid; i < MG * kC * DSUB; i += kKmThreads) s_sum[i] = 0.f;
    for (int i = tid; i < MG * kC; i += kKmThreads) s_w[i] = 0.f;
    __syncthreads();
    const int64_t t0 = (int64_t)blockIdx.x * kKmChunk;
    const int64_t t1 = (t0 + kKmChunk < n_tok) ? t0 + kKmChunk : n_tok;
    const int mi = tid % MG;                                    // fixed per thread: the stride below is a multiple of MG
    const int m = m0 + mi;
    const half_t* cbm = cb + ((int64_t)g * M + m) * kC * DSUB;
    double obj = 0.0;
    for (int64_t t = t0 + tid / MG; t < t1; t += kKmThreads / MG) {
        const int64_t row = bg * n_tok + t;
        const float wt = w[row];
        const int c = codes[row * M + m];
        float xv[DSUB], cv[DSUB];
        if constexpr (DSUB == 4) {
            const half4_t a = *(const half4_t*)(x + row * kD + m * DSUB);
            const half4_t b = *(const half4_t*)(cbm + c * DSUB);
#pragma unroll
            for (int e = 0; e < 4; ++e) { xv[e] = (float)a[e]; cv[e] = (float)b[e]; }
        } else {
#pragma unroll
            for (int u = 0; u < DSUB / 8; ++u) {
                const half8_t a = *(const half8_t*)(x + row * kD + m * DSUB + 8 * u);
                const half8_t b = *(const half8_t*)(cbm + c * DSUB + 8 * u);
#pragma unroll
                for (int e = 0; e < 8; ++e) { xv[8 * u + e] = (float)a[e]; cv[8 * u + e] = (float)b[e]; }
            }
        }
        float dist = 0.f;
        float* acc = &s_sum[mi * DSUB * kC + c];                // [mi][e][c]: for one e the lanes' banks follow their codes
#pragma unroll
        for (int e = 0; e < DSUB; ++e) {
            const float df = xv[e] - cv[e];
            dist = fmaf(df, df, dist);
            atomicAdd(acc + e * kC, wt * xv[e]);
        }
        atomicAdd(&s_w[mi * kC + c], wt);
        obj += (double)wt * (double)dist;
    }
    // objective: lanes with the same mi (lane % MG, since 64 % MG == 0) combine, then one atomic per wave and sub-space
#pragma unroll
    for (int off = MG; off < 64; off <<= 1) obj += __shfl_xor(obj, off, 64);
    if ((tid & 63) < MG && objective) unsafeAtomicAdd(objective + (int64_t)g * M + m, obj);
    __syncthreads();
    float* gs = sums + ((int64_t)g * M + m0) * kC * DSUB;
    for (int i = tid; i < MG * kC * DSUB; i += kKmThreads) {   // i = (mi, c, e) in the global [m][c][e] order
        const int e = i % DSUB, c = (i / DSUB) % kC, mi2 = i / (DSUB * kC);
        const float v = s_sum[(mi2 * DSUB + e) * kC + c];
        if (v != 0.f) unsafeAtomicAdd(gs + i, v);
    }
    float* gw = wsum + ((int64_t)g * M + m0) * kC;
    for (int i = tid; i < MG * kC; i += kKmThreads) {
        const float v = s_w[i];
        if (v != 0.f) unsafeAtomicAdd(gw + i, v);
    }
}

// 4096 centroids, codes packed 12 bits each (code m at bits 12 m .. 12 m + 11 of the token's row).  A thread owns one
// 16-byte chunk (8 channels) of a token row: tid % 16 = chunk, 16 tokens per pass of the workgroup.
template <int DSUB>
__global__ __launch_bounds__(kKmThreads) void km_accumulate12(
    const half_t* __restrict__ x, const float* __restrict__ w, const uint8_t* __restrict__ codes,
    const half_t* __restrict__ cb, int64_t n_tok, int Hkv, float* __restrict__ sums, float* __restrict__ wsum,
    double* __restrict__ objective)
{
    constexpr int M = kD / DSUB, LPM = DSUB / 8, CB = 3 * M / 2, NC = 4096;
    const int tid = threadIdx.x;
    const int64_t bg = blockIdx.y;
    const int g = (int)(bg % Hkv);
    const int u = tid & 15;                                      // chunk of the row: channels 8 u .. 8 u + 7
    const int m = u / LPM, part = u % LPM;                       // sub-space and the chunk's place inside it
    const int64_t t0 = (int64_t)blockIdx.x * kKmChunk;
    const int64_t t1 = (t0 + kKmChunk < n_tok) ? t0 + kKmChunk : n_tok;
    const half_t* cbm = cb + ((int64_t)g * M + m) * NC * DSUB;
    float* sm = sums + ((int64_t)g * M + m) * NC * DSUB;
    float* wm = wsum + ((int64_t)g * M + m) * NC;
    double obj = 0.0;
    for (int64_t t = t0 + (tid >> 4); t < t1; t += kKmThreads / 16) {
        const int64_t row = bg * n_tok + t;
        const float wt = w[row];
        // the 12 bits of code m start at bit 12 m of the row: two bytes hold them
        const uint8_t* cr = codes + row * CB + (12 * m >> 3);
        const uint32_t two = (uint32_t)cr[0] | ((uint32_t)cr[1] << 8);
        const int c = (int)((two >> ((12 * m) & 7)) & 0xFFFu);
        const half8_t a = *(const half8_t*)(x + row * kD + 8 * u);
        const half8_t b = *(const half8_t*)(cbm + (int64_t)c * DSUB + 8 * part);
        float dist = 0.f;
        float* acc = sm + (int64_t)c * DSUB + 8 * part;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float xv = (float)a[e];
            const float df = xv - (float)b[e];
            dist = fmaf(df, df, dist);
            const float v = wt * xv;
            if (v != 0.f) unsafeAtomicAdd(acc + e, v);
        }
        if (part == 0 && wt != 0.f) unsafeAtomicAdd(wm + c, wt);
        obj += (double)wt * (double)dist;
    }
    // objective of sub-space m: the LPM chunk lanes and the four token slots of a wave (lanes u, u+16, u+32, u+48)
#pragma unroll
    for (int off = 1; off < LPM; off <<= 1) obj += __shfl_xor(obj, off, 64);
    obj += __shfl_xor(obj, 16, 64);
    obj += __shfl_xor(obj, 32, 64);
    if ((tid & 63) < 16 && part == 0 && objective) unsafeAtomicAdd(objective + (int64_t)g * M + m, obj);
}

// weighted means; a centroid without assigned weight keeps its old value
template <int DSUB>
__global__ __launch_bounds__(256) void km_finalize(const float* __restrict__ sums, const float* __restrict__ wsum,
                                                   const half_t* __restrict__ cb_in, half_t* __restrict__ cb_out,
                                                   float* __restrict__ wsum_out, int64_t n_centroids)
{
    // a thread takes up to 8 channels of one centroid, so that neighbouring threads touch neighbouring memory
    constexpr int PER = DSUB < 8 ? DSUB : 8, PARTS = DSUB / PER;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t / PARTS;                                         // (g, m, c) flattened
    const int part = (int)(t % PARTS);
    if (i >= n_centroids) return;
    const float ws = wsum[i];
    if (wsum_out && part == 0) wsum_out[i] = ws;
#pragma unroll
    for (int e = PER * part; e < PER * part + PER; ++e)
        cb_out[i * DSUB + e] = ws > 0.f ? (half_t)(sums[i * DSUB + e] / ws) : cb_in[i * DSUB + e];
}

struct KmPlan {
    size_t off_sums, off_wsum, off_obj, total;
};

KmPlan km_plan(const Geom& g)
{
    KmPlan p;
    size_t off = 0;
    p.off_sums = off; off += align_up((size_t)g.Hkv * kD * g.C * sizeof(float));      // M * d_sub = D
    p.off_wsum = off; off += align_up((size_t)g.Hkv * g.M * g.C * sizeof(float));
    p.off_obj = off;  off += align_up((size_t)g.Hkv * g.M * sizeof(double));
    p.total = off;
    return p;
}

template <int DSUB, bool WIDE>
hipError_t launch_t(const Geom& g, const half_t* x, const float* w, int64_t n_tok, const half_t* cb_in, half_t* cb_out,
                    const uint8_t* codes, float* wsum_out, double* objective, char* ws, hipStream_t st)
{
    const KmPlan p = km_plan(g);
    float* sums = (float*)(ws + p.off_sums);
    float* wsum = (float*)(ws + p.off_wsum);
    double* obj = objective ? objective : (double*)(ws + p.off_obj);
    const int64_t n_zero = (int64_t)(p.total / 4);
    hipLaunchKernelGGL(km_zero, dim3((unsigned)((n_zero + 255) / 256)), dim3(256), 0, st, (uint32_t*)ws, n_zero);
    if (objective)
        hipLaunchKernelGGL(km_zero, dim3((unsigned)((g.Hkv * g.M * 2 + 255) / 256)), dim3(256), 0, st, (uint32_t*)objective,
                           (int64_t)g.Hkv * g.M * 2);
    if (n_tok > 0) {
        if constexpr (WIDE) {
            dim3 grid((unsigned)((n_tok + kKmChunk - 1) / kKmChunk), (unsigned)(g.B * g.Hkv));
            hipLaunchKernelGGL(km_accumulate12<DSUB>, grid, dim3(kKmThreads), 0, st, x, w, codes, cb_in, n_tok, g.Hkv, sums,
                               wsum, obj);
        } else {
            dim3 grid((unsigned)((n_tok + kKmChunk - 1) / kKmChunk), (unsigned)(g.B * g.Hkv), kKmGroups);
            hipLaunchKernelGGL(km_accumulate<DSUB>, grid, dim3(kKmThreads), 0, st, x, w, codes, cb_in, n_tok, g.Hkv, sums,
                               wsum, obj);
        }
    }
    const int64_t n_cen = (int64_t)g.Hkv * g.M * g.C;
    const int64_t n_fin = n_cen * (DSUB < 8 ? 1 : DSUB / 8);
    hipLaunchKernelGGL(km_finalize<DSUB>, dim3((unsigned)((n_fin + 255) / 256)), dim3(256), 0, st, sums, wsum, cb_in,
                       cb_out, wsum_out, n_cen);
    return hipGetLastError();
}

}  // namespace

size_t kmeans_workspace_bytes(const Geom& g) { return km_plan(g).total; }

// codes [B][Hkv][n_tok][code bytes] must already hold the assignment of x to cb_in
hipError_t launch_kmeans_update(const Geom& g, const half_t* x, const float* w, int64_t n_tok, const half_t* cb_in,
                                half_t* cb_out, const uint8_t* codes, float* wsum_out, double* objective, void* ws,
                                hipStream_t st)
{
    if (g.C == 4096) {
        if (g.d == 32) return launch_t<32, true>(g, x, w, n_tok, cb_in, cb_out, codes, wsum_out, objective, (char*)ws, st);
        return launch_t<16, true>(g, x, w, n_tok, cb_in, cb_out, codes, wsum_out, objective, (char*)ws, st);
    }
    switch (g.d) {
    case 4: return launch_t<4, false>(g, x, w, n_tok, cb_in, cb_out, codes, wsum_out, objective, (char*)ws, st);
    case 8: return launch_t<8, false>(g, x, w, n_tok, cb_in, cb_out, codes, wsum_out, objective, (char*)ws, st);
    default: return launch_t<16, false>(g, x, w, n_tok, cb_in, cb_out, codes, wsum_out, objective, (char*)ws, st);
    }
}

}  // namespace antkv
