// VQ encode: nearest-centroid assignment of K / V sub-vectors (paper Sec. 3.1).
//
// argmin_c ||x - c||^2 = argmax_c (x.c - ||c||^2 / 2).  The comparison value of 32 tokens against 32 centroids
// comes out of the matrix core directly: v_mfma_f32_32x32x16_f16 has 16 k slots, the sub-vector fills 4 or 8 of them
// and three more carry -||c||^2/2 split into three fp16 terms (hi + mid + lo reproduce the fp32 value) against ones
// on the token side; for 16-channel sub-vectors the three terms go through a second MFMA.  Centroids sit on the MFMA
// row axis and tokens on the column axis: a lane then owns one token and sees 16 centroid scores per tile in its
// accumulator registers, which makes the running arg-max a per-lane affair with compile-time centroid indices
// (done on groups of 8 scores, see below).  Lanes l and l+32 hold complementary centroid subsets of the
// same token and are combined once per sub-space.  Ties resolve to the lower centroid index (strict '>'
// while indices ascend, explicit index compare across the lane pair).
//
// One workgroup keeps the whole codebook of one KV head in LDS in operand layout -- the centroids (64 KB fp16) and the
// three norm terms per centroid -- and walks over 32-token blocks; token sub-vectors are loaded straight from global
// memory in MFMA operand layout (L1 absorbs the row re-use across sub-spaces).
#include "common.h"

namespace antkv {

namespace {

// maxima of finite scores; this file is compiled with -fno-honor-nans so that the chains below become
// v_max3_f32 / v_max_f32 without NaN canonicalisation of the MFMA results
__device__ __forceinline__ float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
__device__ __forceinline__ float max2f(float a, float b) { return fmaxf(a, b); }

constexpr int kEncThreads = 1024;
constexpr int kEncWaves = kEncThreads / 64;
constexpr float kNormScale = 16.f;     // see the norm terms in the kernel: sub-vector norms up to ||c||^2 = 2.09e6 stay finite

// LDS layout per sub-vector width (halfs per centroid): the A operand of a lane is 8 consecutive halfs
//   d = 4   one array  [M][256][8]  = {c0..c3, n_hi, n_mid, n_lo, 0}: lanes 0-31 read it, lanes 32-63 multiply by zero
//   d = 8   two arrays [M][256][8]: the centroid (lanes 0-31) and {n_hi, n_mid, n_lo, 0 x 5} (lanes 32-63)
//   d = 16  the centroid [M][256][16] (lanes 0-31 the first 8 channels, lanes 32-63 the rest) and a second array
//           [M][256][4] = {n_hi, n_mid, n_lo, 0} for the second MFMA
constexpr size_t enc_lds_bytes(int d) { return d == 16 ? 65536 + 16384 : 131072; }

template <int DSUB>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(
    const half_t* __restrict__ x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
    const half_t* __restrict__ cb, uint8_t* __restrict__ codes, int64_t N_cap, int64_t token_offset,
    int B, int Hkv, int wg_per_head)
{
    constexpr int M = kD / DSUB;
    extern __shared__ uint4_t smem[];
    half_t* s_a = (half_t*)smem;                                   // first array (see above)
    half_t* s_n = s_a + (DSUB == 16 ? 32768 : (DSUB == 8 ? 32768 : 0));   // norm terms (d = 4: inside s_a)
    const int tid = threadIdx.x;
    const int g = blockIdx.x / wg_per_head, wgi = blockIdx.x % wg_per_head;

    // ---- the codebook of this KV head into LDS, with -||c||^2/2 as three fp16 terms per centroid
    const half_t* src = cb + (size_t)g * 32768;
    for (int e = tid; e < M * kC; e += kEncThreads) {              // e = (sub-space, centroid)
        float cf[DSUB];
        if constexpr (DSUB == 4) {
            const half4_t v = *(const half4_t*)(src + e * 4);
#pragma unroll
            for (int t = 0; t < 4; ++t) cf[t] = (float)v[t];
        } else {
#pragma unroll
            for (int u = 0; u < DSUB / 8; ++u) {
                const half8_t v = *(const half8_t*)(src + e * DSUB + 8 * u);
#pragma unroll
                for (int t = 0; t < 8; ++t) cf[8 * u + t] = (float)v[t];
                if constexpr (DSUB == 8) *(half8_t*)(s_a + e * 8) = v;
                else *(half8_t*)(s_a + e * 16 + 8 * u) = v;
            }
        }
        float nn = 0.f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) nn = fmaf(cf[t], cf[t], nn);
        // (stored divided by kNormScale and met by kNormScale in the token operand: a power of two, so nothing is
        // rounded, and -||c||^2/2 stays finite in fp16 up to ||c||^2 = 2 * 65504 * kNormScale)
        const float nv = -0.5f * nn * (1.0f / kNormScale);
        const half_t n_hi = (half_t)nv;
        const float r1 = nv - (float)n_hi;
        const half_t n_mid = (half_t)r1;
        const half_t n_lo = (half_t)(r1 - (float)n_mid);
        const half_t z = (half_t)0.f;
        if constexpr (DSUB == 4) {
            *(half8_t*)(s_a + e * 8) = half8_t{(half_t)cf[0], (half_t)cf[1], (half_t)cf[2], (half_t)cf[3], n_hi, n_mid, n_lo, z};
        } else if constexpr (DSUB == 8) {
            *(half8_t*)(s_n + e * 8) = half8_t{n_hi, n_mid, n_lo, z, z, z, z, z};
        } else {
            *(half4_t*)(s_n + e * 4) = half4_t{n_hi, n_mid, n_lo, z};
        }
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const half_t one = (half_t)kNormScale, zero = (half_t)0.f;        // multiplies the three norm terms
    const half8_t ones3 = {one, one, one, zero, zero, zero, zero, zero};
    const half8_t zeros = {zero, zero, zero, zero, zero, zero, zero, zero};
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
            // token operand: the sub-vector in the k slots of the centroid, ones against the three norm terms
            half8_t bx = zeros, bn = zeros;
            if constexpr (DSUB == 4) {
                if (h == 0) {
                    const half4_t v = *(const half4_t*)(xr + m * 4);
                    bx = half8_t{v[0], v[1], v[2], v[3], one, one, one, zero};
                }
            } else if constexpr (DSUB == 8) {
                bx = ones3;
                if (h == 0) bx = *(const half8_t*)(xr + m * 8);
            } else {
                bx = *(const half8_t*)(xr + m * 16 + 8 * h);
                if (h == 0) bn = ones3;
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
            // this lane's A-operand row of tile 0; a tile is 32 rows further
            const half_t* ap;
            const half_t* an = s_n + (m * kC + n) * 4;                                  // d = 16 only
            if constexpr (DSUB == 4) ap = s_a + (m * kC + n) * 8;
            else if constexpr (DSUB == 8) ap = (h == 0 ? s_a : s_n) + (m * kC + n) * 8;
            else ap = s_a + (m * kC + n) * 16 + 8 * h;
            constexpr int kTileStride = 32 * (DSUB == 16 ? 16 : 8);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const half8_t a = *(const half8_t*)(ap + t * kTileStride);
                float16_t acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bx, acc, 0, 0, 0);
                if constexpr (DSUB == 16) {
                    const half4_t a4 = *(const half4_t*)(an + t * 32 * 4);
                    const half8_t a2 = {a4[0], a4[1], a4[2], a4[3], zero, zero, zero, zero};
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, bn, acc, 0, 0, 0);
                }
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
    const size_t shmem = enc_lds_bytes(g.d);
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
