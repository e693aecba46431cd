// Keys stored before RoPE (paper Sec. 3.3, last paragraph: the pre-RoPE strategy): a decode step needs
// q . RoPE_{pos0 + j}(K_eff[j]) with K_eff[j] the FP16 anchor row or the centroids of the token's codes (Sec. 2.1: the
// rotary embedding that turns K into K~).  The kernels here work out that product for every token and head of the group
// and leave it in the caller's workspace; the rotated keys themselves are never written.  The decode kernels then take
// their scores from there instead of from a lookup table.
//
// RoPE rotates channel pair i = 0 .. 63 by the angle pos * base^(-2 i / 128); the pair is (2 i, 2 i + 1) (style 0) or
// (i, i + 64) (style 1).  Angles of absolute positions are reduced in fp64 (pos * theta reaches 10^5 rad and more).
#include "common.h"

namespace antkv {

namespace {

// cos, sin of pos * theta with the product reduced to (-pi, pi] in fp64
__device__ __forceinline__ void angle_of(int64_t pos, double theta, float& c, float& s)
{
    const double two_pi = 6.283185307179586476925286766559, inv_two_pi = 0.15915494309189533576888376337251;
    const double a = (double)pos * theta;
    const float r = (float)fma(-two_pi, rint(a * inv_two_pi), a);   // (a turn more or less at a tie of the rounding is the same angle)
    __sincosf(r, &s, &c);
    // the fast pair above is good to about 1e-6 on the reduced range; one Newton-like renormalisation keeps |(c, s)| = 1
    const float n = rsqrtf(c * c + s * s);
    c *= n;
    s *= n;
}

// ---- one-byte codes ------------------------------------------------------------------------------------------------
// q . RoPE_p(k) for the group's four heads, in log2 units (scale * log2 e folded into q): 16 bytes per token and KV
// head.  Layout: [B][Hkv][n_pad / 4][4 heads][4 tokens] fp32 with n_pad = N rounded up to 64,
// the form in which the decode kernel's lanes (one head, four consecutive tokens each) read it with one 16-byte load.
// A workgroup (12 waves: as many as the LDS leaves room for) owns a token range of one (sequence, KV head) and keeps
// in LDS the K codebook code-major with rows padded to 272 bytes (a lane = a token, and all lanes read the same 16-byte
// column of different rows: without the padding that is one bank group) and cos / sin of delta * theta_i for
// delta = 0 .. 127, a token's offset inside its 128-token tile (lane l has the tokens l and l + 64 of the tile).
// With p = (tile base) + delta, q . R_p(k) = (R_{-base} q) . (R_delta k): per tile, lane i rotates the four heads'
// pair i of q back by the base angle (worked out exactly: fp64 reduction) and leaves it in the wave's LDS area; per
// token and pair that leaves one rotation by a tabulated angle and the four dot products.  The rotated query is read
// once per pair for both tokens of a lane: those broadcast reads are what the kernel spends most LDS time on.  fp32
// arithmetic on the fp16 inputs.
constexpr int kRsThreads = 768, kRsWaves = kRsThreads / 64;
constexpr int kRsTile = 128;                                           // tokens per wave and step
constexpr int kRsRow = 272;                                            // bytes of a padded codebook row in LDS
constexpr int kRsTab = 0, kRsDelta = kRsTab + kC * kRsRow;             // [256][272]; then [64 pairs][64 lanes] x (cos, sin of l, of l + 64)
constexpr int kRsQ = kRsDelta + 64 * 64 * 16;                          // [waves][64 pairs][x of 4 heads, y of 4 heads] fp32
constexpr int kRsLds = kRsQ + kRsWaves * 64 * 32;
static_assert(kRsLds <= 163840, "LDS budget of one CU");

struct RsParams {
    const half_t* q;                   // [B][Hq][128]
    const uint8_t* codes;              // [B][Hkv][N_cap][M]
    const half_t* cb;                  // [Hkv][M][256][d]
    const int32_t* idx;                // K anchor list and rows (pre-RoPE), for the second kernel
    const half_t* rows;
    float* scores;                     // [B][Hkv][n_pad / 4][4][4]
    int64_t N, N_cap, n_pad, pos0, chunk;
    int k, Hq, Hkv, G, S;
    int plain;                         // score layout [B][Hkv][N][4 heads] (the 12-bit kernels' form) instead of the grouped one
    float c1;
    double log2_base;
};

template <int DSUB, int STYLE>
__global__ __launch_bounds__(kRsThreads) void rope_scores_kernel(const RsParams p)
{
    constexpr int M = kD / DSUB;
    extern __shared__ uint4_t rs_smem[];
    char* smem = (char*)rs_smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bg = blockIdx.x / p.S, sp = blockIdx.x % p.S;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int64_t t0 = (int64_t)sp * p.chunk;                          // a multiple of 128
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
    if (t0 >= t1) return;
    // ---- tables
    {
        const half_t* cbg = p.cb + (size_t)g * 32768;
        for (int ci = tid; ci < 4096; ci += kRsThreads) {              // 16-byte chunk w16 (8 channels) of centroid row `code`
            const int code = ci >> 4, w16 = ci & 15;
            uint4_t v;
            if constexpr (DSUB == 8) {
                v = ((const uint4_t*)cbg)[w16 * 256 + code];
            } else if constexpr (DSUB == 16) {
                v = ((const uint4_t*)cbg)[((w16 >> 1) * 256 + code) * 2 + (w16 & 1)];
            } else {
                const uint2_t lo = ((const uint2_t*)cbg)[(2 * w16) * 256 + code], hi = ((const uint2_t*)cbg)[(2 * w16 + 1) * 256 + code];
                v = uint4_t{lo[0], lo[1], hi[0], hi[1]};
            }
            *(uint4_t*)(smem + kRsTab + code * kRsRow + w16 * 16) = v;
        }
        for (int e = tid; e < 64 * 64; e += kRsThreads) {
            const int pair = e >> 6, l = e & 63;
            const double th = exp2(-(2.0 * pair / kD) * p.log2_base);
            float c0, s0, c1, s1;
            angle_of(l, th, c0, s0);
            angle_of(l + 64, th, c1, s1);
            ((float4_t*)(smem + kRsDelta))[e] = float4_t{c0, s0, c1, s1};
        }
    }
    // lane i: pair i of the four heads' queries, scaled
    const int my_ca = STYLE == 0 ? 2 * lane : lane, my_cb = STYLE == 0 ? 2 * lane + 1 : lane + kD / 2;
    float qa[4], qb[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        qa[h] = qb[h] = 0.f;
        if (h < p.G) {
            const half_t* qh = p.q + ((int64_t)b * p.Hq + g * p.G + h) * kD;
            qa[h] = (float)qh[my_ca] * p.c1;
            qb[h] = (float)qh[my_cb] * p.c1;
        }
    }
    __syncthreads();
    const double theta = exp2(-(2.0 * lane / kD) * p.log2_base);       // lane i looks after pair i's base angle
    const uint8_t* ck = p.codes + (int64_t)bg * p.N_cap * M;
    float4_t* s_qr = (float4_t*)(smem + kRsQ + wave * (64 * 32));       // this wave's rotated queries: [pair][x, y]
    const int64_t n_tiles = (t1 - t0 + kRsTile - 1) / kRsTile;
    for (int64_t tile = wave; tile < n_tiles; tile += kRsWaves) {
        const int64_t tok0 = t0 + tile * kRsTile;
        const bool second = tok0 + 64 < t1;                            // the tile's second half exists (uniform)
        uint32_t cw[2][M / 4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t tok = tok0 + 64 * u + lane;
            const int64_t ltok = tok < p.N ? tok : p.N - 1;
            if constexpr (M == 8) {
                const uint2_t a = *(const uint2_t*)(ck + ltok * M);
                cw[u][0] = a[0]; cw[u][1] = a[1];
            } else {
#pragma unroll
                for (int i = 0; i < M / 16; ++i) {
                    const uint4_t a = *(const uint4_t*)(ck + ltok * M + 16 * i);
#pragma unroll
                    for (int e = 0; e < 4; ++e) cw[u][4 * i + e] = a[e];
                }
            }
        }
        {
            float bc, bs;
            angle_of(p.pos0 + tok0, theta, bc, bs);
            float4_t qx, qy;                                              // R_{-base} (qa, qb)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                qx[h] = qa[h] * bc + qb[h] * bs;
                qy[h] = qb[h] * bc - qa[h] * bs;
            }
            __builtin_amdgcn_wave_barrier();                              // the previous tile's readers are done
            s_qr[2 * lane] = qx;
            s_qr[2 * lane + 1] = qy;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        // (the angle table never changes, but read through an address the compiler cannot follow: it would otherwise
        // keep all 256 values of a lane across the tiles, in scratch memory)
        uint32_t delta_off = (uint32_t)kRsDelta + 16u * (uint32_t)lane;
        asm volatile("" : "+v"(delta_off));
        const char* s_delta = smem + delta_off;
        auto code_of_sub = [&](int u, int m) -> uint32_t { return (cw[u][m >> 2] >> (8 * (m & 3))) & 0xffu; };
        // 8 channels (chunk w16 of a token's de-quantised row) as floats
        auto chunk = [&](int u, int w16, float (&v)[8]) {
            uint4_t r;
            if constexpr (DSUB == 4) {
                const uint2_t lo = *(const uint2_t*)(smem + kRsTab + code_of_sub(u, 2 * w16) * kRsRow + w16 * 16);
                const uint2_t hi = *(const uint2_t*)(smem + kRsTab + code_of_sub(u, 2 * w16 + 1) * kRsRow + w16 * 16 + 8);
                r = uint4_t{lo[0], lo[1], hi[0], hi[1]};
            } else {
                r = *(const uint4_t*)(smem + kRsTab + code_of_sub(u, DSUB == 8 ? w16 : (w16 >> 1)) * kRsRow + w16 * 16);
            }
            const half8_t hv = __builtin_bit_cast(half8_t, r);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (float)hv[e];
        };
        float4_t acc[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};
        // channel pair `pair` of both tokens: (ka, kb) of token l in k0, of token l + 64 in k1
        auto pair_term = [&](int pair, float ka0, float kb0, float ka1, float kb1) {
            const float4_t d = *(const float4_t*)(s_delta + pair * 1024);
            const float4_t qx = s_qr[2 * pair], qy = s_qr[2 * pair + 1];
            const float xr0 = ka0 * d[0] - kb0 * d[1], yr0 = ka0 * d[1] + kb0 * d[0];
            const float xr1 = ka1 * d[2] - kb1 * d[3], yr1 = ka1 * d[3] + kb1 * d[2];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                acc[0][h] = fmaf(qx[h], xr0, fmaf(qy[h], yr0, acc[0][h]));
                acc[1][h] = fmaf(qx[h], xr1, fmaf(qy[h], yr1, acc[1][h]));
            }
        };
        if constexpr (STYLE == 0) {
#pragma unroll
            for (int w16 = 0; w16 < 16; ++w16) {
                float v0[8], v1[8];
                chunk(0, w16, v0);
                chunk(1, w16, v1);
#pragma unroll
                for (int j = 0; j < 4; ++j) pair_term(4 * w16 + j, v0[2 * j], v0[2 * j + 1], v1[2 * j], v1[2 * j + 1]);
            }
        } else {
#pragma unroll
            for (int w16 = 0; w16 < 8; ++w16) {
                float va0[8], vb0[8], va1[8], vb1[8];
                chunk(0, w16, va0);
                chunk(0, w16 + 8, vb0);
                chunk(1, w16, va1);
                chunk(1, w16 + 8, vb1);
#pragma unroll
                for (int e = 0; e < 8; ++e) pair_term(8 * w16 + e, va0[e], vb0[e], va1[e], vb1[e]);
            }
        }
        // lane = token, acc = its four heads  ->  lane 4 u + h = head h of tokens 4 u .. 4 u + 3 (a 4 x 4 transposition
        // inside every quad of lanes); a half tile's 64 float4 are then consecutive.  Tokens past N (the tail of the last
        // 64 tokens) carry the last token's score: finite, and never used.
        const int r0 = lane & 3;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            float4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = r0 ^ r;                                 // lane ^ r is token k of the quad and wants this lane's head k
                float send = acc[u][0];
#pragma unroll
                for (int h = 1; h < 4; ++h) send = (k == h) ? acc[u][h] : send;
                const float got = r == 0 ? send : __shfl_xor(send, r, 64);
#pragma unroll
                for (int h = 0; h < 4; ++h) v[h] = (k == h) ? got : v[h];
            }
            if (u == 0 || second) ((float4_t*)p.scores)[(int64_t)bg * p.n_pad + tok0 + 64 * u + lane] = v;
        }
    }
}

// the K anchor tokens: the same score from the FP16 row (pre-RoPE), a wave per kRowsPerWave entries, lane = pair; replaces
// the score that the kernel above wrote from the codes
constexpr int kRowsPerWave = 8;
template <int STYLE>
__global__ __launch_bounds__(256) void rope_row_scores_kernel(const RsParams p)
{
    const int lane = threadIdx.x & 63;
    const int bg = blockIdx.y, b = bg / p.Hkv, g = bg % p.Hkv;
    const int ca = STYLE == 0 ? 2 * lane : lane, cb = STYLE == 0 ? 2 * lane + 1 : lane + kD / 2;
    const double theta = exp2(-(2.0 * lane / kD) * p.log2_base);
    float qa[4], qb[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        qa[h] = qb[h] = 0.f;
        if (h < p.G) {
            const half_t* qh = p.q + ((int64_t)b * p.Hq + g * p.G + h) * kD;
            qa[h] = (float)qh[ca] * p.c1;
            qb[h] = (float)qh[cb] * p.c1;
        }
    }
    const int e0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kRowsPerWave;
    if (e0 >= p.k) return;
    // all entries' loads are issued before the first is used (entries past the list repeat the last one and are not written)
    int64_t tok[kRowsPerWave];
    float ka[kRowsPerWave], kb[kRowsPerWave];
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
        const int e = e0 + i < p.k ? e0 + i : p.k - 1;
        tok[i] = p.idx[(int64_t)bg * p.k + e];
        const half_t* r = p.rows + ((int64_t)bg * p.k + e) * kD;
        ka[i] = (float)r[ca];
        kb[i] = (float)r[cb];
    }
#pragma unroll
    for (int i = 0; i < kRowsPerWave; ++i) {
        float c, s;
        angle_of(p.pos0 + tok[i], theta, c, s);
        const float xr = ka[i] * c - kb[i] * s, yr = ka[i] * s + kb[i] * c;
        // four sums over the wave in seven exchanges: the first two halve what a lane carries (the lanes of bit 5 = a
        // take heads 2 a, 2 a + 1; of those, the lanes of bit 4 = c take head 2 a + c), the rest add up 16 lanes
        float v[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) v[h] = qa[h] * xr + qb[h] * yr;
        const bool up5 = lane & 32, up4 = lane & 16;
        const float k0 = (up5 ? v[2] : v[0]) + __shfl_xor(up5 ? v[0] : v[2], 32, 64);
        const float k1 = (up5 ? v[3] : v[1]) + __shfl_xor(up5 ? v[1] : v[3], 32, 64);
        float sum = (up4 ? k1 : k0) + __shfl_xor(up4 ? k0 : k1, 16, 64);
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if ((lane & 15) == 0 && e0 + i < p.k) {                           // lane 16 h holds head h
            if (p.plain) p.scores[((int64_t)bg * p.N + tok[i]) * 4 + (lane >> 4)] = sum;
            else p.scores[((int64_t)bg * p.n_pad + (tok[i] & ~3LL)) * 4 + 4 * (lane >> 4) + (tok[i] & 3)] = sum;
        }
    }
}

// ---- the same scores for 12-bit codes (4096 centroids; sub-vectors of 32 or 16 channels) ------------------------------
// The K codebook (1 MB per KV head) stays in the L2, so a token's centroids are fetched the way the 12-bit decode kernel
// fetches its values: 16 lanes per token, each lane the 16 bytes (or two pieces of 8) that hold its four channel pairs,
// four tokens per wave and step.  A lane therefore always works on the same four pairs: it keeps the four heads' pairs
// of q, rotated back by the tile's base angle, in registers (the base angles of the 64 pairs are worked out by the wave,
// lane = pair, and passed through LDS), takes cos / sin of delta * theta from the table [delta][pair] in LDS, and the
// four partial dot products are added up over the 16 lanes.  Output: [B][Hkv][N][4 heads] fp32.
constexpr int kR12Threads = 1024, kR12Waves = kR12Threads / 64;
constexpr int kR12Delta = 0;                                           // [64 deltas][64 pairs] float2
constexpr int kR12Base = kR12Delta + 64 * 64 * 8;                      // [waves][64 pairs] float2
constexpr int kR12Codes = kR12Base + kR12Waves * 64 * 8;               // [waves][64 tokens][8 codes] uint16
constexpr int kR12Lds = kR12Codes + kR12Waves * 64 * 16;

template <int DS, int STYLE>
__global__ __launch_bounds__(kR12Threads) void rope_scores12_kernel(const RsParams p)
{
    constexpr int M = kD / DS, CB = 3 * M / 2, kC12 = 4096;
    extern __shared__ uint4_t rs_smem[];
    char* smem = (char*)rs_smem;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bg = blockIdx.x / p.S, sp = blockIdx.x % p.S;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
    if (t0 >= t1) return;
    for (int e = tid; e < 64 * 64; e += kR12Threads) {
        const int delta = e >> 6, pair = e & 63;
        float c, s;
        angle_of(delta, exp2(-(2.0 * pair / kD) * p.log2_base), c, s);
        ((float2*)(smem + kR12Delta))[e] = float2{c, s};
    }
    const int li = lane & 15, grp = lane >> 4;
    // the lane's pairs 4 li .. 4 li + 3: channels (2 pr, 2 pr + 1), i.e. the 16 bytes from channel 8 li on, or (pr, pr + 64),
    // i.e. 8 bytes from channel 4 li on and 8 bytes from channel 64 + 4 li on
    float qa[4][4], qb[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int pr = 4 * li + j;
        const int ca = STYLE == 0 ? 2 * pr : pr, cb = STYLE == 0 ? 2 * pr + 1 : pr + kD / 2;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            qa[j][h] = qb[j][h] = 0.f;
            if (h < p.G) {
                const half_t* qh = p.q + ((int64_t)b * p.Hq + g * p.G + h) * kD;
                qa[j][h] = (float)qh[ca] * p.c1;
                qb[j][h] = (float)qh[cb] * p.c1;
            }
        }
    }
    __syncthreads();
    const double theta = exp2(-(2.0 * lane / kD) * p.log2_base);       // lane i looks after pair i's base angle
    const uint8_t* ck = p.codes + (int64_t)bg * p.N_cap * CB;
    const char* cbg = (const char*)(p.cb + (size_t)g * M * kC12 * DS);
    float2* s_base = (float2*)(smem + kR12Base) + wave * 64;
    uint16_t* s_codes = (uint16_t*)(smem + kR12Codes) + wave * (64 * 8);
    // byte offsets of the lane's pieces inside a centroid, and their sub-spaces
    constexpr int kPieces = STYLE == 0 ? 1 : 2;
    int piece_m[kPieces], piece_off[kPieces];
    if constexpr (STYLE == 0) {
        piece_m[0] = (8 * li) / DS; piece_off[0] = ((8 * li) % DS) * 2;
    } else {
        piece_m[0] = (4 * li) / DS; piece_off[0] = ((4 * li) % DS) * 2;
        piece_m[1] = (64 + 4 * li) / DS; piece_off[1] = ((64 + 4 * li) % DS) * 2;
    }
    const int64_t n_tiles = (t1 - t0 + 63) >> 6;
    for (int64_t tile = wave; tile < n_tiles; tile += kR12Waves) {
        const int64_t tok0 = t0 + tile * 64;
        {
            float bc, bs;
            angle_of(p.pos0 + tok0, theta, bc, bs);
            // this lane's token of the tile: its codes, unpacked (two 12-bit codes in three bytes), go to LDS for the 16
            // lanes that will work on the token
            const int64_t ltok = tok0 + lane < p.N ? tok0 + lane : p.N - 1;
            const uint8_t* row = ck + ltok * CB;                         // (rows are 2-byte aligned only)
            uint32_t cw[CB / 2];
#pragma unroll
            for (int i = 0; i < CB / 2; ++i) cw[i] = *(const uint16_t*)(row + 2 * i);
            uint32_t code[M];
#pragma unroll
            for (int i = 0; i < M / 2; ++i) {                             // bytes 3 i .. 3 i + 2 = 16-bit words 3 i / 2 ..
                const uint32_t w24 = (i & 1) ? ((cw[3 * i / 2] >> 8) | (cw[3 * i / 2 + 1] << 8)) : (cw[3 * i / 2] | (cw[3 * i / 2 + 1] << 16));
                code[2 * i] = w24 & 0xfffu;
                code[2 * i + 1] = (w24 >> 12) & 0xfffu;
            }
            __builtin_amdgcn_wave_barrier();                              // the previous tile's readers are done
            s_base[lane] = float2{bc, bs};
            if constexpr (M == 4) {
                *(uint2_t*)(s_codes + lane * 8) = uint2_t{code[0] | (code[1] << 16), code[2] | (code[3] << 16)};
            } else {
                *(uint4_t*)(s_codes + lane * 8) = uint4_t{code[0] | (code[1] << 16), code[2] | (code[3] << 16),
                                                          code[4] | (code[5] << 16), code[6] | (code[7] << 16)};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        float qx[4][4], qy[4][4];                                         // R_{-base} (qa, qb) of the lane's pairs
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 cs = s_base[4 * li + j];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                qx[j][h] = qa[j][h] * cs.x + qb[j][h] * cs.y;
                qy[j][h] = qb[j][h] * cs.x - qa[j][h] * cs.y;
            }
        }
        uint32_t delta_off = (uint32_t)kR12Delta + 32u * (uint32_t)li;   // (read through an address the compiler cannot follow:
        asm volatile("" : "+v"(delta_off));                               //  the table would otherwise be kept in registers or scratch)
#pragma unroll 4
        for (int step = 0; step < 16; ++step) {
            const int tl = 4 * step + grp;                                // the token's place in the tile = its delta
            const uint16_t* cr = s_codes + tl * 8;
            float ka[4], kb[4];
            auto code_of_sub = [&](int m) -> uint32_t { return cr[m]; };
            if constexpr (STYLE == 0) {
                const uint32_t code = code_of_sub(piece_m[0]);
                const half8_t v = *(const half8_t*)(cbg + ((size_t)(piece_m[0] * kC12 + code) * DS) * 2 + piece_off[0]);
#pragma unroll
                for (int j = 0; j < 4; ++j) { ka[j] = (float)v[2 * j]; kb[j] = (float)v[2 * j + 1]; }
            } else {
                const uint32_t code_a = code_of_sub(piece_m[0]), code_b = code_of_sub(piece_m[1]);
                const half4_t va = *(const half4_t*)(cbg + ((size_t)(piece_m[0] * kC12 + code_a) * DS) * 2 + piece_off[0]);
                const half4_t vb = *(const half4_t*)(cbg + ((size_t)(piece_m[1] * kC12 + code_b) * DS) * 2 + piece_off[1]);
#pragma unroll
                for (int j = 0; j < 4; ++j) { ka[j] = (float)va[j]; kb[j] = (float)vb[j]; }
            }
            const float4_t d01 = *(const float4_t*)(smem + delta_off + (uint32_t)tl * 512u);
            const float4_t d23 = *(const float4_t*)(smem + delta_off + (uint32_t)tl * 512u + 16u);
            const float dc[4] = {d01[0], d01[2], d23[0], d23[2]}, ds[4] = {d01[1], d01[3], d23[1], d23[3]};
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float xr = ka[j] * dc[j] - kb[j] * ds[j], yr = ka[j] * ds[j] + kb[j] * dc[j];
#pragma unroll
                for (int h = 0; h < 4; ++h) acc[h] = fmaf(qx[j][h], xr, fmaf(qy[j][h], yr, acc[h]));
            }
            // sums over the 16 lanes of the token (rotations inside a row of 16 lanes: no LDS traffic)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                acc[h] += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, acc[h]), 0x128, 0xf, 0xf, true));   // row_ror:8
                acc[h] += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, acc[h]), 0x124, 0xf, 0xf, true));   // row_ror:4
                acc[h] += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, acc[h]), 0x122, 0xf, 0xf, true));   // row_ror:2
                acc[h] += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, acc[h]), 0x121, 0xf, 0xf, true));   // row_ror:1
            }
            const int64_t tok = tok0 + tl;
            if (li == 0 && tok < p.N) ((float4_t*)p.scores)[(int64_t)bg * p.N + tok] = float4_t{acc[0], acc[1], acc[2], acc[3]};
        }
    }
}

}  // namespace

hipError_t launch_rope_scores(const Geom& g, const half_t* q, float scale, const uint8_t* codes_k, int64_t N, int64_t N_cap,
                              const half_t* cb_k, const int32_t* idx_k, const half_t* rows_k, int64_t k_k, double rope_base,
                              int rope_style, int64_t pos0, float* scores_out, hipStream_t st)
{
    if (N == 0 || g.B == 0) return hipSuccess;
    RsParams p;
    p.q = q; p.codes = codes_k; p.cb = cb_k; p.idx = idx_k; p.rows = rows_k; p.scores = scores_out;
    p.n_pad = (N + 63) / 64 * 64;
    p.plain = g.C != kC;
    p.N = N; p.N_cap = N_cap; p.pos0 = pos0; p.k = (int)k_k; p.Hq = g.Hq; p.Hkv = g.Hkv; p.G = g.G;
    p.c1 = scale * kLog2e; p.log2_base = log2(rope_base);
    const int64_t bg = (int64_t)g.B * g.Hkv;
    int64_t S = (256 + bg - 1) / bg;                                  // about one workgroup per CU
    const int64_t max_S = (N + 1023) / 1024;
    if (S > max_S) S = max_S;
    if (S < 1) S = 1;
    int64_t chunk = ((N + S - 1) / S + kRsTile - 1) / kRsTile * kRsTile;
    p.chunk = chunk;
    p.S = (int)((N + chunk - 1) / chunk);
    const dim3 grid((unsigned)(bg * p.S));
    hipError_t e = hipSuccess;
#define ANTKV_RS12(DS, STY)                                                                                                \
    do {                                                                                                                   \
        static const hipError_t once = hipFuncSetAttribute((const void*)rope_scores12_kernel<DS, STY>,                     \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kR12Lds);           \
        if (once != hipSuccess) return once;                                                                               \
        hipLaunchKernelGGL((rope_scores12_kernel<DS, STY>), grid, dim3(kR12Threads), kR12Lds, st, p);                      \
    } while (0)
#define ANTKV_RS(DS, STY)                                                                                                  \
    do {                                                                                                                   \
        static const hipError_t once = hipFuncSetAttribute((const void*)rope_scores_kernel<DS, STY>,                       \
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRsLds);            \
        if (once != hipSuccess) return once;                                                                               \
        hipLaunchKernelGGL((rope_scores_kernel<DS, STY>), grid, dim3(kRsThreads), kRsLds, st, p);                          \
    } while (0)
    if (g.C != kC) {
        if (g.d == 32) { if (rope_style == 0) ANTKV_RS12(32, 0); else ANTKV_RS12(32, 1); }
        else { if (rope_style == 0) ANTKV_RS12(16, 0); else ANTKV_RS12(16, 1); }
    }
    else if (g.d == 4) { if (rope_style == 0) ANTKV_RS(4, 0); else ANTKV_RS(4, 1); }
    else if (g.d == 8) { if (rope_style == 0) ANTKV_RS(8, 0); else ANTKV_RS(8, 1); }
    else { if (rope_style == 0) ANTKV_RS(16, 0); else ANTKV_RS(16, 1); }
#undef ANTKV_RS
#undef ANTKV_RS12
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (k_k > 0) {
        const dim3 grid2((unsigned)((k_k + 4 * kRowsPerWave - 1) / (4 * kRowsPerWave)), (unsigned)bg);
        if (rope_style == 0) hipLaunchKernelGGL(rope_row_scores_kernel<0>, grid2, dim3(256), 0, st, p);
        else hipLaunchKernelGGL(rope_row_scores_kernel<1>, grid2, dim3(256), 0, st, p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace antkv
