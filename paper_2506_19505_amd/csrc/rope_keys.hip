// Keys stored before RoPE (paper Sec. 3.3, last paragraph: the pre-RoPE strategy): before a decode step uses them, every
// key of the cache is brought to its position, K_rot[j] = RoPE_{pos0 + j}(K_eff[j]) with K_eff[j] the FP16 anchor row
// or the centroids of the token's codes (Sec. 2.1: the rotary embedding that turns K into K~).  The rotated keys are
// written as FP16 rows, one per token, together with the identity index list; decode attention then takes them as a
// K anchor list that covers every token.
//
// RoPE rotates channel pair i = 0 .. 63 by the angle pos * base^(-2 i / 128); the pair is (2 i, 2 i + 1) (style 0) or
// (i, i + 64) (style 1).  One lane per pair.  The angle of a run's first token is reduced in fp64 (pos * theta reaches
// 10^5 rad), the following tokens of the run advance by one fp32 complex multiplication with e^{i theta} each.
#include "common.h"

namespace antkv {

namespace {

constexpr int kRunTokens = 16;         // tokens a 64-lane group rotates one after another
constexpr int kGroups = 4;             // groups per workgroup

struct RkParams {
    const uint8_t* codes;              // [B][Hkv][N_cap][code_bytes]
    const half_t* cb;                  // [Hkv][M][C][d]
    const int32_t* idx;                // [B][Hkv][k] positions of the FP16 rows
    const half_t* rows;                // [B][Hkv][k][128] FP16 rows, before RoPE
    half_t* out;                       // [B][Hkv][N][128]
    int32_t* iota;                     // [B][Hkv][N]: iota[j] = j
    int64_t N, N_cap, pos0;
    int k, Hkv, d, M, C, code_bytes, style;
    double log2_base;
};

__device__ __forceinline__ void pair_channels(int style, int i, int& ca, int& cb)
{
    if (style == 0) { ca = 2 * i; cb = 2 * i + 1; } else { ca = i; cb = i + kD / 2; }
}
// cos, sin of pos * theta with the product reduced to (-pi, pi] in fp64
__device__ __forceinline__ void angle_of(int64_t pos, double theta, float& c, float& s)
{
    const double two_pi = 6.283185307179586476925286766559;
    const double a = (double)pos * theta;
    const float r = (float)(a - two_pi * rint(a / two_pi));
    __sincosf(r, &s, &c);
    // the fast pair above is good to about 1e-6 on the reduced range; one Newton-like renormalisation keeps |(c, s)| = 1
    const float n = rsqrtf(c * c + s * s);
    c *= n;
    s *= n;
}
__device__ __forceinline__ int code_of(const RkParams& p, const uint8_t* row, int m)
{
    if (p.C == kC) return row[m];
    const uint8_t* t = row + 3 * (m >> 1);            // two 12-bit codes in three bytes
    return (m & 1) ? ((t[1] >> 4) | (t[2] << 4)) : (t[0] | ((t[1] & 0xf) << 8));
}

__global__ __launch_bounds__(64 * kGroups) void rope_dequant_kernel(const RkParams p)
{
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int bg = blockIdx.y, g = bg % p.Hkv;
    const int64_t j0 = ((int64_t)blockIdx.x * kGroups + grp) * kRunTokens;
    if (j0 >= p.N) return;
    int ca, cb;
    pair_channels(p.style, lane, ca, cb);
    const double theta = exp2(-(2.0 * lane / kD) * p.log2_base);
    float c, s, cd, sd;
    angle_of(p.pos0 + j0, theta, c, s);
    angle_of(1, theta, cd, sd);
    const int ma = ca / p.d, ea = ca % p.d, mb = cb / p.d, eb = cb % p.d;
    const half_t* cba = p.cb + ((size_t)g * p.M + ma) * p.C * p.d + ea;
    const half_t* cbb = p.cb + ((size_t)g * p.M + mb) * p.C * p.d + eb;
    for (int t = 0; t < kRunTokens && j0 + t < p.N; ++t) {
        const int64_t j = j0 + t;
        const uint8_t* row = p.codes + ((int64_t)bg * p.N_cap + j) * p.code_bytes;
        const float a = (float)cba[(size_t)code_of(p, row, ma) * p.d];
        const float b = (float)cbb[(size_t)code_of(p, row, mb) * p.d];
        half_t* o = p.out + ((int64_t)bg * p.N + j) * kD;
        o[ca] = (half_t)(a * c - b * s);
        o[cb] = (half_t)(a * s + b * c);
        if (lane == 0) p.iota[(int64_t)bg * p.N + j] = (int32_t)j;
        const float cn = c * cd - s * sd;
        s = s * cd + c * sd;
        c = cn;
    }
}

// the FP16 anchor rows replace the rotated centroids of their tokens
__global__ __launch_bounds__(64 * kGroups) void rope_rows_kernel(const RkParams p)
{
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int bg = blockIdx.y;
    const int e = blockIdx.x * kGroups + grp;
    if (e >= p.k) return;
    int ca, cb;
    pair_channels(p.style, lane, ca, cb);
    const double theta = exp2(-(2.0 * lane / kD) * p.log2_base);
    const int64_t j = p.idx[(int64_t)bg * p.k + e];
    float c, s;
    angle_of(p.pos0 + j, theta, c, s);
    const half_t* r = p.rows + ((int64_t)bg * p.k + e) * kD;
    const float a = (float)r[ca], b = (float)r[cb];
    half_t* o = p.out + ((int64_t)bg * p.N + j) * kD;
    o[ca] = (half_t)(a * c - b * s);
    o[cb] = (half_t)(a * s + b * c);
}

}  // namespace

hipError_t launch_rope_keys(const Geom& g, const uint8_t* codes_k, int64_t N, int64_t N_cap, const half_t* cb_k,
                            const int32_t* idx_k, const half_t* rows_k, int64_t k_k, double rope_base, int rope_style,
                            int64_t pos0, half_t* rows_out, int32_t* iota_out, hipStream_t st)
{
    if (N == 0 || g.B == 0) return hipSuccess;
    RkParams p;
    p.codes = codes_k; p.cb = cb_k; p.idx = idx_k; p.rows = rows_k; p.out = rows_out; p.iota = iota_out;
    p.N = N; p.N_cap = N_cap; p.pos0 = pos0; p.k = (int)k_k; p.Hkv = g.Hkv; p.d = g.d; p.M = g.M; p.C = g.C;
    p.code_bytes = g.code_bytes; p.style = rope_style; p.log2_base = log2(rope_base);
    const int64_t runs = (N + kRunTokens - 1) / kRunTokens;
    dim3 grid((unsigned)((runs + kGroups - 1) / kGroups), (unsigned)(g.B * g.Hkv));
    hipLaunchKernelGGL(rope_dequant_kernel, grid, dim3(64 * kGroups), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (k_k > 0) {
        dim3 grid2((unsigned)((k_k + kGroups - 1) / kGroups), (unsigned)(g.B * g.Hkv));
        hipLaunchKernelGGL(rope_rows_kernel, grid2, dim3(64 * kGroups), 0, st, p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace antkv
