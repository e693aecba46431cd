// VQ encode: nearest-centroid assignment of K / V sub-vectors (paper Sec. 3.1).
//
// argmin_c ||x - c||^2 = argmax_c (x.c - ||c||^2 / 2).  The x.c contraction of 32 tokens against 32
// centroids runs on one v_mfma_f32_32x32x8_f16 whose accumulator is pre-loaded with -||c||^2/2, so the
// matrix core emits the comparison value directly.  Centroids sit on the MFMA row axis and tokens on
// the column axis: a lane then owns one token and sees 16 centroid scores per tile in its accumulator
// registers, which makes the running arg-max a per-lane affair with compile-time centroid indices
// (done on groups of 8 scores, see below).  Lanes l and l+32 hold complementary centroid subsets of the
// same token and are combined once per sub-space.  Ties resolve to the lower centroid index (strict '>'
// while indices ascend, explicit index compare across the lane pair).
//
// One workgroup keeps the whole codebook of one KV head (64 KB fp16) plus the -||c||^2/2 table in LDS
// and walks over 32-token blocks; token sub-vectors are loaded straight from global memory in MFMA
// operand layout (8 bytes per lane, L1 absorbs the row re-use across sub-spaces).
#include "common.h"

namespace antkv {

namespace {

// maxima of finite scores; this file is compiled with -fno-honor-nans so that the chains below become
// v_max3_f32 / v_max_f32 without NaN canonicalisation of the MFMA results
__device__ __forceinline__ float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
__device__ __forceinline__ float max2f(float a, float b) { return fmaxf(a, b); }

constexpr int kEncThreads = 512;
constexpr int kEncWaves = kEncThreads / 64;

template <int DSUB>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(
    const half_t* __restrict__ x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
    const half_t* __restrict__ cb, uint8_t* __restrict__ codes, int64_t N_cap, int64_t token_offset,
    int B, int Hkv, int wg_per_head)
{
    constexpr int M = kD / DSUB;
    extern __shared__ uint4_t smem[];
    half_t* s_cb = (half_t*)smem;            // [M][256][DSUB] fp16, 64 KB
    float* s_nrm = (float*)(s_cb + 32768);   // [M][256] : -||c||^2 / 2
    const int tid = threadIdx.x;
    const int g = blockIdx.x / wg_per_head, wgi = blockIdx.x % wg_per_head;

    const uint4_t* src = (const uint4_t*)(cb + (size_t)g * 32768);
    for (int i = tid; i < 4096; i += kEncThreads) smem[i] = src[i];
    __syncthreads();
    for (int e = tid; e < M * kC; e += kEncThreads) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) {
            const float v = (float)s_cb[e * DSUB + t];
            s = fmaf(v, v, s);
        }
        s_nrm[e] = -0.5f * s;
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const int64_t blocks_per_b = (n_tok + 31) / 32;
    const int64_t total = (int64_t)B * blocks_per_b;
    for (int64_t unit = (int64_t)wgi * kEncWaves + wave; unit < total; unit += (int64_t)wg_per_head * kEncWaves) {
        const int64_t b = unit / blocks_per_b;
        const int64_t tok = (unit % blocks_per_b) * 32 + n;
        const bool valid = tok < n_tok;
        const half_t* xr = x + b * xs_b + (int64_t)g * xs_h + (valid ? tok : n_tok - 1) * xs_t;
        uint8_t* dst = codes + (((int64_t)b * Hkv + g) * N_cap + token_offset + (valid ? tok : 0)) * M;

#pragma unroll 1
        for (int m4 = 0; m4 < M / 4; ++m4) {
          uint32_t word = 0u;
#pragma unroll
          for (int mm = 0; mm < 4; ++mm) {
            const int m = 4 * m4 + mm;
            half4_t b0 = {0, 0, 0, 0}, b1 = {0, 0, 0, 0};
            if (DSUB == 4) {
                if (h == 0) b0 = *(const half4_t*)(xr + m * 4);
            } else if (DSUB == 8) {
                b0 = *(const half4_t*)(xr + m * 8 + 4 * h);
            } else {
                b0 = *(const half4_t*)(xr + m * 16 + 4 * h);
                b1 = *(const half4_t*)(xr + m * 16 + 8 + 4 * h);
            }
            // Running maximum over groups of 8 candidates (registers 8*hf .. 8*hf+7 of a tile).  The group maximum
            // comes from a max3 tree; when a group raises the running maximum (strictly, so the lowest group wins
            // ties) its id and its 8 scores are kept.  Which of the 8 it was is settled once per sub-space, from
            // the kept scores, in ascending index order: 15 VALU ops per 8 candidates instead of 24.
            float best = -3.0e38f;
            int gid = 0;
            float keep[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) keep[e] = -3.0e38f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int crow = m * kC + 32 * t;
                half4_t a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
                if (DSUB == 4) {
                    if (h == 0) a0 = *(const half4_t*)(s_cb + (crow + n) * 4);
                } else if (DSUB == 8) {
                    a0 = *(const half4_t*)(s_cb + (crow + n) * 8 + 4 * h);
                } else {
                    a0 = *(const half4_t*)(s_cb + (crow + n) * 16 + 4 * h);
                    a1 = *(const half4_t*)(s_cb + (crow + n) * 16 + 8 + 4 * h);
                }
                float16_t acc;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4_t nv = *(const float4_t*)(s_nrm + crow + 8 * q + 4 * h);
                    acc[4 * q + 0] = nv[0];
                    acc[4 * q + 1] = nv[1];
                    acc[4 * q + 2] = nv[2];
                    acc[4 * q + 3] = nv[3];
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a0, b0, acc, 0, 0, 0);
                if (DSUB == 16) acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a1, b1, acc, 0, 0, 0);
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const int r0 = 8 * hf;
                    const float m0 = max3f(acc[r0 + 0], acc[r0 + 1], acc[r0 + 2]);
                    const float m1 = max3f(acc[r0 + 3], acc[r0 + 4], acc[r0 + 5]);
                    const float m2 = max3f(m0, m1, acc[r0 + 6]);
                    const float m3 = max2f(m2, acc[r0 + 7]);
                    const bool better = m3 > best;
                    best = better ? m3 : best;
                    gid = better ? (2 * t + hf) : gid;
#pragma unroll
                    for (int e = 0; e < 8; ++e) keep[e] = better ? acc[r0 + e] : keep[e];
                }
            }
            // the winning group's centroids are 32 t + 16 hf + 8 j2 + 4 h + e (j2 < 2, e < 4), ascending in j = 4 j2 + e
            int bidx;
            {
                const int c_base = 32 * (gid >> 1) + 16 * (gid & 1) + 4 * h;
                float fbest = keep[0];
                int jb = 0;
#pragma unroll
                for (int j = 1; j < 8; ++j) {
                    const bool better = keep[j] > fbest;
                    fbest = better ? keep[j] : fbest;
                    jb = better ? j : jb;
                }
                bidx = c_base + 8 * (jb >> 2) + (jb & 3);
            }
            const float ob = __shfl_xor(best, 32, 64);
            const int oi = __shfl_xor(bidx, 32, 64);
            if (ob > best || (ob == best && oi < bidx)) bidx = oi;
            word |= (uint32_t)bidx << (8 * mm);
          }
          if (valid && h == 0) *(uint32_t*)(dst + 4 * m4) = word;
        }
    }
}

}  // namespace

hipError_t launch_encode(const Geom& g, const half_t* x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
                         const half_t* cb, uint8_t* codes, int64_t N_cap, int64_t token_offset, hipStream_t st)
{
    if (n_tok == 0 || g.B == 0) return hipSuccess;
    const int64_t blocks = (int64_t)g.B * ((n_tok + 31) / 32);
    int64_t wgph = (blocks + kEncWaves - 1) / kEncWaves;
    const int64_t cap = (256 + g.Hkv - 1) / g.Hkv;   // about one workgroup per CU in total
    if (wgph > cap) wgph = cap;
    if (wgph < 1) wgph = 1;
    const size_t shmem = 65536 + (size_t)g.M * kC * 4;
    dim3 grid((unsigned)(g.Hkv * wgph)), block(kEncThreads);
#define ANTKV_ENC(DS)                                                                                           \
    do {                                                                                                        \
        hipError_t e = hipFuncSetAttribute((const void*)encode_kernel<DS>,                                      \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);             \
        if (e != hipSuccess) return e;                                                                          \
        hipLaunchKernelGGL(encode_kernel<DS>, grid, block, shmem, st, x, xs_b, xs_h, xs_t, n_tok, cb, codes,    \
                           N_cap, token_offset, g.B, g.Hkv, (int)wgph);                                         \
    } while (0)
    if (g.d == 4) ANTKV_ENC(4);
    else if (g.d == 8) ANTKV_ENC(8);
    else ANTKV_ENC(16);
#undef ANTKV_ENC
    return hipGetLastError();
}

}  // namespace antkv
