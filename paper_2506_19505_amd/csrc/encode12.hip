// VQ encode for the 12-bit codebooks (paper Sec. 3.1 with the 4096-centroid settings of Sec. 4: d32, "0.375 bit", and
// d16, "0.75 bit"): nearest of 4096 centroids for each 32- or 16-channel sub-vector, the M = 4 or 8 codes of a token
// row packed into 6 or 12 bytes.
//
// argmin_c ||x - c||^2 = argmax_c (x.c - ||c||^2 / 2).  A 1 MB codebook per KV head does not fit LDS, so centroid
// tiles come straight from global memory (L2; the four waves of a workgroup walk the same tiles, so L1 serves three
// of them; a wave uses each tile for both of its 32-token groups) and only the -||c||^2/2 table of the current
// sub-space (16 KB) is kept in LDS.
//   level 1  per 32 tokens x 32 centroids: v_mfma_f32_32x32x16_f16 (one per 16 channels) with centroids on the row
//            axis and tokens on the column axis, accumulator pre-loaded with -||c||^2/2.  A lane owns one token and 16 of the 32
//            centroid scores; it keeps the best score and the index of the tile it came from (a max3 tree, one
//            compare and two selects per tile, i.e. under one VALU instruction per candidate).
//   level 2  the lane recomputes the 16 scores of its best tile with packed dot products (v_dot2_f32_f16), in
//            ascending centroid order with a strict '>' (ties go to the lower index); lanes l and l+32, which
//            hold complementary centroid subsets of the same token, are then combined.
// Both levels are fp32-accurate; they may order two centroids differently only when their scores agree to
// fp32 rounding.
#include "common.h"

namespace antkv {

namespace {

constexpr int kE12Threads = 256;
constexpr int kE12Tokens = 256;          // tokens per workgroup: 4 waves x 2 groups of 32
constexpr int kC12 = 4096;

__device__ __forceinline__ float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

__device__ __forceinline__ float dot8(const half8_t& a, const half8_t& b, float acc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = {a[2 * i], a[2 * i + 1]}, y = {b[2 * i], b[2 * i + 1]};
        acc = __builtin_amdgcn_fdot2(x, y, acc, false);
    }
    return acc;
}

// kD12 = sub-vector width (32 or 16)
template <int kD12>
__global__ __launch_bounds__(kE12Threads) void encode12_kernel(
    const half_t* __restrict__ x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
    const half_t* __restrict__ cb, uint8_t* __restrict__ codes, int64_t N_cap, int64_t token_offset, int Hkv)
{
    constexpr int kM12 = kD / kD12;                                 // 4 or 8 sub-spaces
    constexpr int NU = kD12 / 8;                                    // 16-byte chunks of a sub-vector
    constexpr int NS = kD12 / 16;                                   // MFMA k-steps
    __shared__ __attribute__((aligned(16))) float s_nrm[kC12];      // -||c||^2 / 2 of the current sub-space
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, kh = lane >> 5;
    const int b = blockIdx.y / Hkv, g = blockIdx.y % Hkv;
    const half_t* xbase = x + (int64_t)b * xs_b + (int64_t)g * xs_h;
    int code[2][kM12];
#pragma unroll
    for (int tg = 0; tg < 2; ++tg)
#pragma unroll
        for (int m = 0; m < kM12; ++m) code[tg][m] = 0;

#pragma unroll 1
    for (int m = 0; m < kM12; ++m) {
        const half_t* cbm = cb + ((int64_t)g * kM12 + m) * kC12 * kD12;
        __syncthreads();                                            // the previous sub-space's table is no longer read
        for (int c = tid; c < kC12; c += kE12Threads) {
            float s = 0.f;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const half8_t v = *(const half8_t*)(cbm + c * kD12 + 8 * u);
                s = dot8(v, v, s);
            }
            s_nrm[c] = -0.5f * s;
        }
        __syncthreads();
        // the wave's two groups of 32 tokens share every centroid tile it loads
        const half_t* xr[2];
        half8_t xb[2][NS];                                          // B operand: k-step s holds channels 16 s + 8 kh .. + 7
        float best[2] = {-3.0e38f, -3.0e38f};
        int best_blk[2] = {0, 0};
#pragma unroll
        for (int tg = 0; tg < 2; ++tg) {
            const int64_t t = (int64_t)blockIdx.x * kE12Tokens + wave * 64 + tg * 32 + n;
            const int64_t tl = t < n_tok ? t : n_tok - 1;
            xr[tg] = xbase + tl * xs_t + m * kD12;
#pragma unroll
            for (int s = 0; s < NS; ++s) xb[tg][s] = *(const half8_t*)(xr[tg] + 16 * s + 8 * kh);
        }
        // A operand of tile blk: centroid 32 blk + n, same channel split; loads run one tile ahead
        const half_t* ap = cbm + n * kD12 + 8 * kh;
        half8_t an[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) an[s] = *(const half8_t*)(ap + 16 * s);
#pragma unroll 2
        for (int blk = 0; blk < kC12 / 32; ++blk) {
            half8_t ac[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s) ac[s] = an[s];
            if (blk + 1 < kC12 / 32) {
#pragma unroll
                for (int s = 0; s < NS; ++s) an[s] = *(const half8_t*)(ap + (blk + 1) * 32 * kD12 + 16 * s);
            }
            float4_t nb[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) nb[qd] = *(const float4_t*)(&s_nrm[blk * 32 + 8 * qd + 4 * kh]);
#pragma unroll
            for (int tg = 0; tg < 2; ++tg) {
                float16_t acc;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)                      // rows 8 qd + 4 kh + e live in acc[4 qd + e]
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[4 * qd + e] = nb[qd][e];
#pragma unroll
                for (int s = 0; s < NS; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(ac[s], xb[tg][s], acc, 0, 0, 0);
                float mx = max3f(acc[0], acc[1], acc[2]);
#pragma unroll
                for (int r = 3; r < 15; r += 2) mx = max3f(mx, acc[r], acc[r + 1]);
                mx = fmaxf(mx, acc[15]);
                if (mx > best[tg]) { best[tg] = mx; best_blk[tg] = blk; }   // strict: an equal later tile does not replace
            }
        }
#pragma unroll
        for (int tg = 0; tg < 2; ++tg) {
            // level 2: the 16 candidates of the best tile, ascending centroid index
            half8_t xf[NU];
#pragma unroll
            for (int u = 0; u < NU; ++u) xf[u] = *(const half8_t*)(xr[tg] + 8 * u);
            float bv = -3.0e38f;
            int bc = 0;
#pragma unroll 4
            for (int r = 0; r < 16; ++r) {
                const int c = best_blk[tg] * 32 + 8 * (r >> 2) + 4 * kh + (r & 3);
                const half_t* cp = cbm + c * kD12;
                float s = s_nrm[c];
#pragma unroll
                for (int u = 0; u < NU; ++u) s = dot8(*(const half8_t*)(cp + 8 * u), xf[u], s);
                if (s > bv) { bv = s; bc = c; }
            }
            // the two halves of the token's candidates: larger score wins, equal scores go to the lower index
            const float ov = __shfl_xor(bv, 32, 64);
            const int oc = __shfl_xor(bc, 32, 64);
            if (ov > bv || (ov == bv && oc < bc)) bc = oc;
            code[tg][m] = bc;
        }
    }
    // the token's 12-bit codes packed little-endian (code m at bits 12 m .. 12 m + 11): 6 or 12 bytes per token
    if (kh == 0) {
#pragma unroll
        for (int tg = 0; tg < 2; ++tg) {
            const int64_t t = (int64_t)blockIdx.x * kE12Tokens + wave * 64 + tg * 32 + n;
            if (t < n_tok) {
                uint16_t* dst = (uint16_t*)(codes + (((int64_t)b * Hkv + g) * N_cap + token_offset + t) * (kM12 * 3 / 2));
#pragma unroll
                for (int q4 = 0; q4 < kM12 / 4; ++q4) {               // four codes fill three 16-bit words
                    const uint32_t c0 = (uint32_t)code[tg][4 * q4], c1 = (uint32_t)code[tg][4 * q4 + 1];
                    const uint32_t c2 = (uint32_t)code[tg][4 * q4 + 2], c3 = (uint32_t)code[tg][4 * q4 + 3];
                    const uint32_t lo = c0 | (c1 << 12) | (c2 << 24);
                    const uint32_t hi = (c2 >> 8) | (c3 << 4);
                    dst[3 * q4 + 0] = (uint16_t)lo;
                    dst[3 * q4 + 1] = (uint16_t)(lo >> 16);
                    dst[3 * q4 + 2] = (uint16_t)hi;
                }
            }
        }
    }
}

}  // namespace

hipError_t launch_encode12(const Geom& g, const half_t* x, int64_t xs_b, int64_t xs_h, int64_t xs_t, int64_t n_tok,
                           const half_t* cb, uint8_t* codes, int64_t N_cap, int64_t token_offset, hipStream_t st)
{
    if (n_tok == 0 || g.B == 0) return hipSuccess;
    dim3 grid((unsigned)((n_tok + kE12Tokens - 1) / kE12Tokens), (unsigned)(g.B * g.Hkv));
    if (g.d == 32)
        hipLaunchKernelGGL(encode12_kernel<32>, grid, dim3(kE12Threads), 0, st, x, xs_b, xs_h, xs_t, n_tok, cb, codes, N_cap,
                           token_offset, g.Hkv);
    else
        hipLaunchKernelGGL(encode12_kernel<16>, grid, dim3(kE12Threads), 0, st, x, xs_b, xs_h, xs_t, n_tok, cb, codes, N_cap,
                           token_offset, g.Hkv);
    return hipGetLastError();
}

}  // namespace antkv
