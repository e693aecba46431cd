// Decode attention over 12-bit VQ codes + FP16 anchors (Attn of paper Sec. 2.1 on the cache of Fig. 2(b), with the
// 4096-centroid codebooks of Sec. 4): one query token per sequence against codes packed 6 bytes per token (d32, four
// sub-spaces) or 12 bytes per token (d16, eight sub-spaces).
//
// With 4096 centroids only the q.centroid table of the K side fits LDS: 128 KB of int16 entries, which is 4 sub-spaces
// x 4096 codes x 4 heads for d32 and 8 sub-spaces x 4096 codes x 2 heads for d16.  There a workgroup with more than two
// heads walks the K codes of its token range twice: first with the table of heads 0 and 1, leaving their scores in a
// scratch array, then with the table of heads 2 and 3, now with the softmax and the value phase for all four heads
// (a token is handled by the same thread both times).  The V codebook (1 MB per KV head) stays in L2, which is
// why workgroup ids are mapped so that KV head g runs on XCD g mod 8 and each XCD's L2 keeps one head's codebook.
//   prologue   table: a small kernel computes the fp32 scores once per (sequence, KV head); each workgroup takes the
//              maximum per head and quantises them to 16-bit fixed point with one scale per head into LDS; bitmaps of the K- and V-anchored tokens of the workgroup's token range (the stream skips
//              them).
//   stream     lane = token: unpack the codes, one table read per sub-space, integer sums, online softmax per
//              64-token tile.  Then the value phase: 16 lanes per token, every lane owns eight output channels,
//              fetches them from the token's V centroid of that sub-space (one 16-byte gather per lane) and adds
//              P_h * v for the workgroup's heads.  Anchored tokens carry weight zero here.
//   anchors    the list entries form tiles of their own (lane = entry), dealt round-robin over the workgroups of the
//              head: score from the FP16 row (or from the table), then the same value phase with the FP16 row (or
//              the centroids) as the source.
//   merge      waves through LDS, workgroups through a partial (max, sum, accumulator) per head and a second
//              small kernel.
#include "common.h"

#include <type_traits>

namespace antkv {

namespace {

constexpr int kT12 = 1024;               // threads
constexpr int kW12 = kT12 / 64;          // waves
constexpr int kC12 = 4096;
constexpr int kNH = 4;                   // head slots of a query group (G <= 4)
constexpr int kChunkMax = 32768;         // tokens per workgroup (bitmaps of 1024 words)
constexpr float kEmptyRef12 = -1.0e4f;   // softmax reference before any token: finite, far above the masked score
constexpr int kLutMax12 = 32767;
constexpr int kTabThreads = 256;
constexpr int tab_blocks(int ds) { return (kD / ds) * kC12 / (kTabThreads * 4); }   // per (sequence, KV head), 4 entries per thread
constexpr int heads_per_table(int ds) { return ds == 32 ? 4 : 2; }                  // heads whose int16 table fits 128 KB
constexpr float kPShift12 = 12.f;        // weights are kept scaled by 2^12 so that small ones stay normal in fp16

struct D12Params {
    const half_t* q;
    const uint8_t *codes_k, *codes_v;
    const half_t *cb_k, *cb_v;
    const int32_t *idx_k, *idx_v;
    const half_t *rows_k, *rows_v;
    float* part;                          // [B][Hq][S][kD + 2]
    const float4_t* tab;                  // [B][Hkv][M][4096] fp32 scores of the four heads, from d12_table_kernel
    const float* tab_amax;                // [B][Hkv][table blocks][4] per-block maxima of |score|
    int64_t N, N_cap;
    int k_k, k_v;
    float c1;
    int Hq, Hkv, G, S, chunk;
    float2* early;                        // [B][Hkv][N] scores of heads 0 and 1 from the first walk (d16 with G > 2), else unused
    const float4_t* given;                // kernels with given scores: [B][Hkv][N] the four heads' scores in log2 units (the K
                                          // codes, the table and the K anchor list are not used then)
};

__device__ __forceinline__ float dot8f(const half8_t& a, const half8_t& b, float acc)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = {a[2 * i], a[2 * i + 1]}, y = {b[2 * i], b[2 * i + 1]};
        acc = __builtin_amdgcn_fdot2(x, y, acc, false);
    }
    return acc;
}

// first position in ascending idx[0..n) whose value is >= target; 64-ary search, every lane returns the same value
__device__ __forceinline__ int lower_bound64(const int32_t* __restrict__ idx, int n, int target, int lane)
{
    int lo = 0, hi = n;                                   // the answer lies in [lo, hi]
    while (hi > lo) {
        const int len = hi - lo;
        const int step = (len + 63) / 64;                 // 64 probes at lo + lane * step cover [lo, hi)
        const int pos = lo + lane * step;
        const bool below = pos < hi && idx[pos] < target;
        const int cnt = (int)__popcll(__ballot(below));   // the list ascends, so these lanes form a prefix
        if (cnt == 0) { hi = lo; break; }
        int nhi = lo + cnt * step;                        // probe cnt is not below the target (or past the end)
        if (nhi > hi) nhi = hi;
        lo = lo + (cnt - 1) * step + 1;                   // probe cnt - 1 is below it
        hi = nhi;                                         // hi - lo <= step - 1 < len: the loop ends
    }
    return lo;
}

// a token's code words: 48 or 96 bits, code m at bits 12 m .. 12 m + 11
template <int DS>
__device__ __forceinline__ void load_cw(const uint8_t* __restrict__ base, int64_t tok, uint32_t (&w)[3])
{
    if constexpr (DS == 32) {
        const uint16_t* s = (const uint16_t*)(base + tok * 6);
        w[0] = (uint32_t)s[0] | ((uint32_t)s[1] << 16);
        w[1] = (uint32_t)s[2];
        w[2] = 0u;
    } else {
        const uint32_t* s = (const uint32_t*)(base + tok * 12);
        w[0] = s[0];
        w[1] = s[1];
        w[2] = s[2];
    }
}

__device__ __forceinline__ uint32_t code12(const uint32_t (&w)[3], int m)
{
    const int bit = 12 * m, d = bit >> 5, sh = bit & 31;       // m is a compile-time constant wherever this is called
    uint32_t v = w[d] >> sh;
    if (sh > 20) v |= w[d + 1] << (32 - sh);
    return v & 0xFFFu;
}

// fp32 table of c1 q_h . centroid for one (sequence, KV head): every workgroup of the decode kernel that works on this
// pair needs the same M x 4096 x 4 values, so they are computed once here (the K codebook is read once instead of
// once per decode workgroup) and only quantised into LDS there.
template <int kD12>
__global__ __launch_bounds__(kTabThreads) void d12_table_kernel(const half_t* __restrict__ q, const half_t* __restrict__ cb_k,
                                                                float c1, int Hq, int Hkv, int G, float4_t* __restrict__ tab,
                                                                float* __restrict__ tab_amax)
{
    __shared__ __attribute__((aligned(16))) half_t s_q[kNH * kD];
    __shared__ float s_red[kTabThreads / 64][kNH];
    constexpr int kM12 = kD / kD12;
    constexpr int kTabBlocks = tab_blocks(kD12);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bg = blockIdx.x, b = bg / Hkv, g = bg % Hkv;
    for (int i = tid; i < kNH * kD; i += kTabThreads)
        s_q[i] = ((i >> 7) < G) ? q[((int64_t)b * Hq + g * G) * kD + i] : (half_t)0.f;
    __syncthreads();
    float amax[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int k = 0; k < 4; ++k) {
        const int e = (blockIdx.y * 4 + k) * kTabThreads + tid;        // entry = (sub-space, code)
        const int m = e / kC12;
        const half_t* cp = cb_k + ((int64_t)g * kM12 * kC12 + e) * kD12;
        half8_t cv[kD12 / 8];
#pragma unroll
        for (int u = 0; u < kD12 / 8; ++u) cv[u] = *(const half8_t*)(cp + 8 * u);
        float4_t o;
#pragma unroll
        for (int h = 0; h < kNH; ++h) {
            float d = 0.f;
#pragma unroll
            for (int u = 0; u < kD12 / 8; ++u) d = dot8f(cv[u], *(const half8_t*)(s_q + h * kD + m * kD12 + 8 * u), d);
            o[h] = d * c1;
            amax[h] = fmaxf(amax[h], fabsf(o[h]));
        }
        tab[(int64_t)bg * kM12 * kC12 + e] = o;
    }
#pragma unroll
    for (int h = 0; h < kNH; ++h) {
        const float wmax = wave_max(amax[h]);
        if (lane == 0) s_red[wave][h] = wmax;
    }
    __syncthreads();
    if (tid < kNH) {
        float a = 0.f;
        for (int w = 0; w < kTabThreads / 64; ++w) a = fmaxf(a, s_red[w][tid]);
        tab_amax[((int64_t)bg * kTabBlocks + blockIdx.y) * kNH + tid] = a;
    }
}

// LDS bytes of decode12_kernel<DS>
constexpr size_t d12_lds(int ds)
{
    return (size_t)128 * 1024 + 1024 * 4 + (size_t)kNH * kD * 2 + 64 * 4 + 16 * 4 + (size_t)kW12 * 64 * kNH * 2 +
           (size_t)kW12 * (kD / ds) * 64 * 2;
}
static_assert(d12_lds(32) <= 160 * 1024 && d12_lds(16) <= 160 * 1024, "LDS budget");

// kD12 = sub-vector width: 32 (four sub-spaces, one table for the four heads of a group) or 16 (eight sub-spaces, a
// table holds two heads)
// GIVEN: the K side's scores come from p.given (keys that are rotated to their position before the product with q have
// no table): no table is loaded, the K codes are not read, the K anchor list is empty and V entries take their token's
// score from p.given.
template <int kD12, bool GIVEN>
__global__ __launch_bounds__(kT12) void decode12_kernel(const D12Params p)
{
    constexpr int kM12 = kD / kD12;                                    // sub-spaces
    constexpr int NHW = kNH;                                           // head slots of the workgroup
    constexpr int NHT = heads_per_table(kD12);                         // heads per table
    constexpr int LPM = kD12 / 8;                                      // value-phase lanes per sub-space
    constexpr int kTabBlocks = tab_blocks(kD12);
    using lut_t = typename std::conditional<NHT == 4, uint2_t, uint32_t>::type;   // NHT x int16
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    lut_t* s_lut = (lut_t*)smem;                                       // [M][4096] entries of NHT x int16 (128 KB)
    uint32_t* s_mk = (uint32_t*)(smem + 128 * 1024);                   // K- or V-anchored tokens of the range, 1024 words
    half_t* s_q = (half_t*)(s_mk + 1024);                              // [NHW][128]
    float* s_red = (float*)(s_q + NHW * kD);                           // 64 floats of scratch
    int* s_misc = (int*)(s_red + 64);                                  // 16 ints
    // this wave's tile: for each pair of tokens (2j, 2j+1) the heads' weights as NHW half2 {P_h(2j), P_h(2j+1)}
    half_t* s_pw = (half_t*)(s_misc + 16) + (threadIdx.x >> 6) * (64 * NHW);
    uint16_t* s_vc = (uint16_t*)((half_t*)(s_misc + 16) + kW12 * 64 * NHW) + (threadIdx.x >> 6) * (kM12 * 64);   // [M][64] V codes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // KV head g on XCD g mod 8: workgroup ids go to the XCDs round-robin
    const int g = blockIdx.x % p.Hkv;
    const int rest = blockIdx.x / p.Hkv;
    const int b = rest / p.S, sp = rest % p.S;
    const int bg = b * p.Hkv + g;
    const int h0 = g * p.G;
    const int nh = p.G;                                                // heads present (<= NHW)
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const int32_t* idx_v = p.idx_v + (int64_t)bg * p.k_v;

    // ---- prologue ----------------------------------------------------------------------------------------------
    if (tid < NHW * kD) s_q[tid] = ((tid >> 7) < nh) ? p.q[((int64_t)b * p.Hq + h0) * kD + tid] : (half_t)0.f;
    s_mk[tid] = 0u;
    if (wave < 4) {                                                    // list ranges that fall into [t0, t1)
        const int32_t* l = (wave < 2) ? idx_k : idx_v;
        const int n = (wave < 2) ? p.k_k : p.k_v;
        const int r = lower_bound64(l, n, (int)((wave & 1) ? t1 : t0), lane);
        if (lane == 0) s_misc[wave] = r;
    }
    __syncthreads();
    const int lo_k = s_misc[0], hi_k = s_misc[1], lo_v = s_misc[2], hi_v = s_misc[3];
    for (int i = lo_k + tid; i < hi_k; i += kT12) {
        const int rel = idx_k[i] - (int)t0;
        atomicOr(&s_mk[rel >> 5], 1u << (rel & 31));
    }
    for (int i = lo_v + tid; i < hi_v; i += kT12) {
        const int rel = idx_v[i] - (int)t0;
        atomicOr(&s_mk[rel >> 5], 1u << (rel & 31));
    }
    constexpr int CB = 3 * kM12 / 2;                                   // code bytes per token
    const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * CB;
    const uint8_t* cv = p.codes_v + (int64_t)bg * p.N_cap * CB;
    const int64_t n_tiles = (t1 - t0 + 63) >> 6;
    // table: the fp32 scores come from d12_table_kernel; one scale per head from the per-block maxima, then 16-bit
    // fixed point into LDS.  Thread t owns entries t + 1024 i.  `walk` selects the NHT heads the table holds.
    float lut_q[NHT];                                                  // table quantum per head (log2 units)
    auto load_table = [&](int walk) {
        float inv_q[NHT];
#pragma unroll
        for (int h = 0; h < NHT; ++h) {
            float a = 0.f;
            for (int k = 0; k < kTabBlocks; ++k) a = fmaxf(a, p.tab_amax[((int64_t)bg * kTabBlocks + k) * kNH + NHT * walk + h]);
            inv_q[h] = a > 0.f ? (float)kLutMax12 / a : 0.f;
            lut_q[h] = a * (1.0f / (float)kLutMax12);
        }
        const float4_t* tb = p.tab + (int64_t)bg * kM12 * kC12;
#pragma unroll 4
        for (int e = tid; e < kM12 * kC12; e += kT12) {
            const float4_t sc = tb[e];
            if constexpr (NHT == 4) {
                int q16[4];
#pragma unroll
                for (int h = 0; h < 4; ++h) q16[h] = (int)rintf(sc[h] * inv_q[h]);
                uint2_t w;
                w[0] = ((uint32_t)q16[0] & 0xFFFFu) | ((uint32_t)q16[1] << 16);
                w[1] = ((uint32_t)q16[2] & 0xFFFFu) | ((uint32_t)q16[3] << 16);
                s_lut[e] = w;
            } else {
                const int qa = (int)rintf((walk ? sc[2] : sc[0]) * inv_q[0]), qb = (int)rintf((walk ? sc[3] : sc[1]) * inv_q[1]);
                s_lut[e] = ((uint32_t)qa & 0xFFFFu) | ((uint32_t)qb << 16);
            }
        }
    };
    // scores of the table's heads for one token
    auto table_scores = [&](const uint32_t (&kw)[3], float (&s)[NHT]) {
        int sum[NHT];
#pragma unroll
        for (int h = 0; h < NHT; ++h) sum[h] = 0;
#pragma unroll
        for (int m = 0; m < kM12; ++m) {
            const lut_t e = s_lut[m * kC12 + code12(kw, m)];
            if constexpr (NHT == 4) {
                sum[0] += (int)(short)(e[0] & 0xFFFFu);
                sum[1] += (int)e[0] >> 16;
                sum[2] += (int)(short)(e[1] & 0xFFFFu);
                sum[3] += (int)e[1] >> 16;
            } else {
                sum[0] += (int)(short)(e & 0xFFFFu);
                sum[1] += (int)e >> 16;
            }
        }
#pragma unroll
        for (int h = 0; h < NHT; ++h) s[h] = (float)sum[h] * lut_q[h];
    };
    const int n_walks = (nh + NHT - 1) / NHT;                          // 1, or 2 for d16 with more than two heads
    float2* early = p.early + (int64_t)bg * p.N;
    const float4_t* given = GIVEN ? p.given + (int64_t)bg * p.N : nullptr;
    if constexpr (!GIVEN) load_table(0);
    __syncthreads();                                                   // table and bitmap are complete
    if (!GIVEN && NHT < NHW && n_walks > 1) {
        // first walk: heads 0 and 1 of every token of the range; tiles go to the waves as in the stream below
        for (int64_t tile = wave; tile < n_tiles; tile += kW12) {
            const int64_t tok = t0 + tile * 64 + lane;
            const int64_t ltok = tok < t1 ? tok : t1 - 1;
            uint32_t kw[3];
            load_cw<kD12>(ck, ltok, kw);
            float s[NHT];
            table_scores(kw, s);
            if (tok < t1) early[tok] = float2{s[0], s[NHT - 1]};
        }
        __syncthreads();                                               // nobody reads the first table any more
        load_table(1);
        __syncthreads();
    }
    const int hb = NHT * (n_walks - 1);                                // head slot of the table's first head

    // ---- per-wave state and the helpers shared by the stream and the anchor tiles
    const half_t* cbv = p.cb_v + (int64_t)g * kM12 * kC12 * kD12;
    // Value phase roles: a group of 16 lanes (grp) takes the tokens t with t mod 4 == grp of a tile, four tokens per
    // gather instruction; lane li of the group owns output channels 8 li .. 8 li + 7, i.e. 16 bytes of the centroid of
    // sub-space li / LPM.  The four groups' accumulators are added up once, before the merge.
    const int grp = lane >> 4, li = lane & 15;
    const int my_m = li / LPM;
    const char* cbv_bytes = (const char*)cbv;
    const uint32_t lane_off = (uint32_t)((my_m * kC12 * kD12 + 8 * (li % LPM)) * 2);    // byte offset of the lane's channels
    float m_ref[NHW], l_lane[NHW], acc[NHW][8];
#pragma unroll
    for (int h = 0; h < NHW; ++h) {
        m_ref[h] = kEmptyRef12;
        l_lane[h] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
    }

    const half_t* cbk = p.cb_k + (int64_t)g * kM12 * kC12 * kD12;
    // scores of all head slots for a token from its codes, outside the stream: the table where it holds every head,
    // else q . centroid summed over the sub-spaces in fp32
    auto code_scores = [&](const uint32_t (&kw)[3], float (&s)[NHW]) {
        if constexpr (NHT == NHW) {
            table_scores(kw, s);
        } else {
#pragma unroll
            for (int h = 0; h < NHW; ++h) s[h] = 0.f;
#pragma unroll
            for (int m = 0; m < kM12; ++m) {
                const half_t* cp = cbk + ((int64_t)m * kC12 + code12(kw, m)) * kD12;
#pragma unroll
                for (int u = 0; u < kD12 / 8; ++u) {
                    const half8_t cvec = *(const half8_t*)(cp + 8 * u);
#pragma unroll
                    for (int h = 0; h < NHW; ++h) s[h] = dot8f(cvec, *(const half8_t*)(s_q + h * kD + m * kD12 + 8 * u), s[h]);
                }
            }
#pragma unroll
            for (int h = 0; h < NHW; ++h) s[h] *= p.c1;
        }
    };
    // move the wave's reference of head h to at least `cand` (uniform); returns nothing, rescales the running state
    auto raise_ref = [&](int h, float cand) {
        if (cand > m_ref[h]) {
            const float alpha = fast_exp2(m_ref[h] - cand);
            l_lane[h] *= alpha;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[h][c] *= alpha;
            m_ref[h] = cand;
        }
    };

    // value phase.  Token t of a tile is step t / 4 of group t mod 4.  A gather covers four steps (16 tokens of the
    // wave); two steps are consumed together: acc[h][ch] += P_h(t) v_ch(t) + P_h(t + 4) v_ch(t + 4) is one
    // v_dot2_f32_f16.  LDS hand-off layouts: codes [sub-space][group][step], weights [group][step pair][head] as half2.
    constexpr int kSteps = 4;                                          // steps per gather batch
    auto gather = [&](int s0, half8_t (&dst)[kSteps]) {               // stream tiles: centroid of the lane's sub-space
        const uint2_t c4 = *(const uint2_t*)(s_vc + my_m * 64 + grp * 16 + s0);    // four steps' codes
#pragma unroll
        for (int e = 0; e < kSteps; ++e) {
            const uint32_t code = (c4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
            dst[e] = *(const half8_t*)(cbv_bytes + (lane_off + code * (uint32_t)(kD12 * 2)));
        }
    };
    auto consume = [&](int s0, const half8_t (&src)[kSteps]) {
#pragma unroll
        for (int e = 0; e < kSteps; e += 2) {
            half_t pj[2 * NHW];                                        // the group's step pair: NHW x {P_h(t), P_h(t + 4)}
            const half_t* pp = s_pw + (grp * 8 + ((s0 + e) >> 1)) * (2 * NHW);
            if constexpr (NHW == 4) {
                const half8_t v8 = *(const half8_t*)pp;
#pragma unroll
                for (int i = 0; i < 8; ++i) pj[i] = v8[i];
            } else {
                const half4_t v4 = *(const half4_t*)pp;
#pragma unroll
                for (int i = 0; i < 4; ++i) pj[i] = v4[i];
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const half2_t vc = {src[e][c], src[e + 1][c]};
#pragma unroll
                for (int h = 0; h < NHW; ++h) {
                    const half2_t ph = {pj[2 * h], pj[2 * h + 1]};
                    acc[h][c] = __builtin_amdgcn_fdot2(ph, vc, acc[h][c], false);
                }
            }
        }
    };
    // online softmax of one tile: raises the wave's references, adds the weights to the lane sums and leaves the
    // heads' weights of every token (fp16, scaled by 2^12) in the wave's LDS area, paired for the dot products
    auto tile_weights = [&](const float (&sc)[NHW], bool off) {
        half_t pw_h[NHW];
#pragma unroll
        for (int h = 0; h < NHW; ++h) {
            const float sh = off ? kNegBig : sc[h];
            raise_ref(h, wave_max(sh));
            const float pw = fast_exp2(sh - m_ref[h] + kPShift12);     // 0 for switched-off lanes, at most 2^12
            l_lane[h] += pw;
            pw_h[h] = (half_t)pw;
        }
        __builtin_amdgcn_wave_barrier();                               // LDS operations of one wave stay in order
#pragma unroll
        for (int h = 0; h < NHW; ++h)                                  // token = lane: group lane % 4, step lane / 4
            s_pw[((lane & 3) * 8 + (lane >> 3)) * (2 * NHW) + 2 * h + ((lane >> 2) & 1)] = pw_h[h];
    };

    // ---- stream ------------------------------------------------------------------------------------------------
    for (int64_t tile = wave; tile < n_tiles; tile += kW12) {
        const int64_t tok = t0 + tile * 64 + lane;
        const int64_t ltok = tok < t1 ? tok : t1 - 1;
        uint32_t kw[3] = {0u, 0u, 0u}, vw[3];
        if constexpr (!GIVEN) load_cw<kD12>(ck, ltok, kw);
        load_cw<kD12>(cv, ltok, vw);
        const int rel = (int)(ltok - t0);
        const uint32_t mbit = (s_mk[rel >> 5] >> (rel & 31)) & 1u;
        const bool masked = tok >= t1 || mbit != 0u;
        float s[NHW];
        if constexpr (GIVEN) {
            const float4_t g4 = given[ltok];
#pragma unroll
            for (int h = 0; h < NHW; ++h) s[h] = g4[h];
        } else if constexpr (NHT == NHW) {
            table_scores(kw, s);
        } else {
            float st[NHT];
            table_scores(kw, st);
            float2 e01 = float2{0.f, 0.f};
            if (hb) e01 = early[ltok];                                  // written by this thread in the first walk
            s[0] = hb ? e01.x : st[0];
            s[1] = hb ? e01.y : st[1];
            s[2] = hb ? st[0] : 0.f;
            s[3] = hb ? st[1] : 0.f;
        }
        tile_weights(s, masked);
#pragma unroll
        for (int m = 0; m < kM12; ++m) s_vc[m * 64 + (lane & 3) * 16 + (lane >> 2)] = (uint16_t)code12(vw, m);
        __builtin_amdgcn_wave_barrier();
        // 16 steps of four tokens; the gathers of the next four steps fly while four are consumed
        half8_t vbuf[2][kSteps];
        gather(0, vbuf[0]);
#pragma unroll
        for (int k = 0; k < 16 / kSteps; ++k) {
            if (k + 1 < 16 / kSteps) gather((k + 1) * kSteps, vbuf[(k + 1) & 1]);
            consume(k * kSteps, vbuf[k & 1]);
        }
    }

    // ---- anchors: the entries of the K list followed by those of the V list form tiles of 64 of their own
    // (lane = entry), dealt round-robin over the S workgroups of the (sequence, KV head) whatever token range an entry
    // falls into, so that anchors clustered in one part of the context do not pile up in one workgroup; whether a
    // K-anchored token is also in the V list (and where), or a V-anchored one also in the K list, is a binary search
    // per lane.  A K entry's score is q . FP16 row, computed by its lane from the row's 16 chunks; a V entry
    // that is not K-anchored scores from the table; a V entry that is also in the K list was handled there.  The value
    // phase is the stream's, with the source of every token (centroid or FP16 row) passed through LDS as a byte offset
    // whose top bit selects the FP16 rows, 32 tokens at a time.  (Anchor tiles come after the stream: with the anchor
    // code first, or with both kinds of tile handed out by one counter, the stream slowed down by more than the
    // overlap gained.)
    const int n_ka = p.k_k, n_va = p.k_v;
    const int n_at = (n_ka + n_va + 63) >> 6;
    const char* rows_v_bytes = (const char*)p.rows_v;
    uint32_t* s_src = (uint32_t*)s_vc;                                 // [M sub-spaces][32 tokens]
    // position of tok in an ascending list, or -1
    auto find = [&](const int32_t* __restrict__ list, int n, int tok) -> int {
        int lo = 0, hi = n;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (list[mid] < tok) lo = mid + 1;
            else hi = mid;
        }
        return (lo < n && list[lo] == tok) ? lo : -1;
    };
    for (int at = sp + p.S * wave; at < n_at; at += p.S * kW12) {
        const int it = at * 64 + lane;
        const bool from_k = it < n_ka, from_v = !from_k && it < n_ka + n_va;
        int i = 0, tok = (int)t0;                                      // a lane without an entry: token t0 with weight 0
        int pos_v = -1;                                                // the token's place in the V list, if it has one
        bool in_k = false;
        if (from_k) { i = it; tok = idx_k[i]; pos_v = find(idx_v, n_va, tok); }
        if (from_v) { i = it - n_ka; tok = idx_v[i]; pos_v = i; in_k = find(idx_k, n_ka, tok) >= 0; }
        const bool in_v = pos_v >= 0;
        const bool active = from_k || (from_v && !in_k);
        float s[NHW];
#pragma unroll
        for (int h = 0; h < NHW; ++h) s[h] = 0.f;
        if (from_k) {
            const half_t* row = p.rows_k + ((int64_t)bg * p.k_k + i) * kD;
#pragma unroll 4
            for (int c = 0; c < kD / 8; ++c) {
                const half8_t kr = *(const half8_t*)(row + 8 * c);
#pragma unroll
                for (int h = 0; h < NHW; ++h) s[h] = dot8f(kr, *(const half8_t*)(s_q + h * kD + 8 * c), s[h]);
            }
#pragma unroll
            for (int h = 0; h < NHW; ++h) s[h] *= p.c1;
        } else if constexpr (GIVEN) {
            const float4_t g4 = given[tok];
#pragma unroll
            for (int h = 0; h < NHW; ++h) s[h] = g4[h];
        } else {
            uint32_t kw[3];
            load_cw<kD12>(ck, tok, kw);
            code_scores(kw, s);
        }
        uint32_t voff[kM12];                                           // byte offset of the token's kD12 channels per sub-space
        if (in_v) {
#pragma unroll
            for (int m = 0; m < kM12; ++m)
                voff[m] = 0x80000000u | (uint32_t)((((int64_t)bg * p.k_v + pos_v) * kD + kD12 * m) * 2);
        } else {
            uint32_t vw[3];
            load_cw<kD12>(cv, tok, vw);
#pragma unroll
            for (int m = 0; m < kM12; ++m) voff[m] = (uint32_t)((m * kC12 + (int)code12(vw, m)) * kD12 * 2);
        }
        tile_weights(s, !active);
        // half tiles of 32 entries: sources [sub-space][group][step], 8 steps per group
        auto gather_a = [&](int s0, half8_t (&dst)[kSteps]) {
            const uint4_t o4 = *(const uint4_t*)(s_src + my_m * 32 + grp * 8 + s0);
#pragma unroll
            for (int e = 0; e < kSteps; ++e) {
                const char* base = (o4[e] & 0x80000000u) ? rows_v_bytes : cbv_bytes;
                dst[e] = *(const half8_t*)(base + (o4[e] & 0x7FFFFFFFu) + 16 * (li % LPM));
            }
        };
#pragma unroll 1
        for (int jb = 0; jb < 64; jb += 32) {
            __builtin_amdgcn_wave_barrier();
            if ((lane >> 5) == (jb >> 5)) {                            // entry = lane: group lane % 4, step (lane % 32) / 4
#pragma unroll
                for (int m = 0; m < kM12; ++m) s_src[m * 32 + (lane & 3) * 8 + ((lane & 31) >> 2)] = voff[m];
            }
            __builtin_amdgcn_wave_barrier();
            half8_t vbuf[2][kSteps];
            gather_a(0, vbuf[0]);
            gather_a(kSteps, vbuf[1]);
            consume((jb >> 2), vbuf[0]);                               // steps jb / 4 .. of the whole tile's weights
            consume((jb >> 2) + kSteps, vbuf[1]);
        }
    }

    // ---- merge the waves, write the workgroup's partial -------------------------------------------------------
    __syncthreads();                                                   // the table is dead: its LDS becomes the merge area
    float* s_m = (float*)smem;                                         // [waves][NHW] references
    float* s_l = s_m + kW12 * NHW;                                     // [waves][NHW] sums
    float* s_acc = s_l + kW12 * NHW;                                   // [waves][NHW][128]
#pragma unroll
    for (int h = 0; h < NHW; ++h) {
        const float lw = wave_sum(l_lane[h]);
        if (lane == 0) { s_m[wave * NHW + h] = m_ref[h]; s_l[wave * NHW + h] = lw; }
#pragma unroll
        for (int c = 0; c < 8; ++c) {                                  // the four groups hold shares of the same channels
            float a = acc[h][c];
            a += __shfl_xor(a, 16, 64);
            a += __shfl_xor(a, 32, 64);
            if (grp == 0) s_acc[(wave * NHW + h) * kD + 8 * li + c] = a;
        }
    }
    __syncthreads();
    if (tid < NHW * kD) {
        const int h = tid >> 7, ch = tid & 127;
        if (h < nh) {
            float m = kEmptyRef12;
            for (int w = 0; w < kW12; ++w) m = fmaxf(m, s_m[w * NHW + h]);
            float l = 0.f, a = 0.f;
            for (int w = 0; w < kW12; ++w) {
                const float f = fast_exp2(s_m[w * NHW + h] - m);
                l = fmaf(s_l[w * NHW + h], f, l);
                a = fmaf(s_acc[(w * NHW + h) * kD + ch], f, a);
            }
            float* dst = p.part + (((int64_t)b * p.Hq + h0 + h) * p.S + sp) * (kD + 2);
            dst[2 + ch] = a;
            if (ch == 0) { dst[0] = m; dst[1] = l; }
        }
    }
}

// merge the S partials of a (sequence, query head) by log-sum-exp and round once to fp16.  The S references and sums go
// through LDS first (one round of loads instead of a chain of S), then every channel thread sums its column with eight
// independent loads in flight.
constexpr int kMergeSlots = 1024;

__global__ __launch_bounds__(kD) void decode12_merge(const float* __restrict__ part, int S, half_t* __restrict__ out)
{
    __shared__ float s_w[kMergeSlots];
    __shared__ float s_tot;
    const int64_t bh = blockIdx.x;
    const int ch = threadIdx.x, lane = ch & 63;
    const float* pb = part + bh * S * (kD + 2);
    if (S > kMergeSlots) {                                             // more slots than the staging holds: plain loops
        float m = kEmptyRef12;
        for (int s = 0; s < S; ++s) m = fmaxf(m, pb[s * (kD + 2)]);
        float l = 0.f, a = 0.f;
        for (int s = 0; s < S; ++s) {
            const float f = fast_exp2(pb[s * (kD + 2)] - m);
            l = fmaf(pb[s * (kD + 2) + 1], f, l);
            a = fmaf(pb[s * (kD + 2) + 2 + ch], f, a);
        }
        out[bh * kD + ch] = (half_t)(l > 0.f ? a / l : 0.f);
        return;
    }
    for (int s = ch; s < S; s += kD) s_w[s] = pb[s * (kD + 2)];
    __syncthreads();
    if (ch < 64) {                                                     // one wave: global reference, slot weights, total sum
        float m = kEmptyRef12;
        for (int s = lane; s < S; s += 64) m = fmaxf(m, s_w[s]);
        m = wave_max(m);
        float l = 0.f;
        for (int s = lane; s < S; s += 64) {
            const float f = fast_exp2(s_w[s] - m);
            s_w[s] = f;
            l = fmaf(pb[s * (kD + 2) + 1], f, l);
        }
        l = wave_sum(l);
        if (lane == 0) s_tot = l;
    }
    __syncthreads();
    float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float* pc = pb + 2 + ch;
    int s = 0;
    for (; s + 8 <= S; s += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = pc[(int64_t)(s + u) * (kD + 2)];
#pragma unroll
        for (int u = 0; u < 8; ++u) a8[u] = fmaf(v[u], s_w[s + u], a8[u]);
    }
    for (; s < S; ++s) a8[0] = fmaf(pc[(int64_t)s * (kD + 2)], s_w[s], a8[0]);
    const float a = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
    const float l = s_tot;
    out[bh * kD + ch] = (half_t)(l > 0.f ? a / l : 0.f);
}

// ---- decode-time Anchor Score on 12-bit codes (Eq. (4) with the single query row over K_eff; Sec. 3.2, last par.) --
// Ranking needs fp32 scores, and an fp32 table of 128 KB holds two heads (d32) or one head (d16), so a workgroup
// walks its token range once per two (one) heads of the group, with that table in LDS: the first walk stores a
// token's scores, the later ones add their heads' shares to them.  A token is always handled by the same thread, so
// these are plain loads and stores in a fixed order (heads ascending) and the result is reproducible.  PASS 0 leaves
// (max, sum of exp2) per head and workgroup; PASS 1 merges them into the log-sum-exp and writes the scores.
struct D12AnsParams {
    const half_t* q;
    const uint8_t* codes_k;
    const int32_t* idx_k;
    const half_t* rows_k;
    const float4_t* tab;
    float* stat_part;                     // [B][Hq][S][2]
    float *ans_k, *ans_v;                 // [B][Hkv][N]
    int64_t N, N_cap;
    int k_k;
    float c1;
    int Hq, Hkv, G, S, chunk;
    uint32_t* hist;                       // optional (pass 1): first-level top-k histograms, [2 B Hkv][2 * kTopkBins], K rows then V rows
};

constexpr size_t kD12AnsLds = (size_t)128 * 1024 + 1024 * 4 + 2 * kD * 4 + (kW12 * 4 + 8) * 4 + 16 * 4 + 2 * kTopkBins * 4;

template <int kD12, int PASS>
__global__ __launch_bounds__(kT12) void d12_ans_kernel(const D12AnsParams p)
{
    constexpr int kM12 = kD / kD12;
    constexpr int NHA = kD12 == 32 ? 2 : 1;                            // heads per walk
    constexpr int CB = 3 * kM12 / 2;
    using lut_t = typename std::conditional<NHA == 2, float2, float>::type;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    lut_t* s_lut = (lut_t*)smem;                                       // [M][4096] scores of this walk's heads
    uint32_t* s_mk = (uint32_t*)(smem + 128 * 1024);                   // K-anchored tokens of the range
    float* s_qf = (float*)(s_mk + 1024);                               // [2][128]
    float* s_red = s_qf + 2 * kD;                                      // [waves][4] + 8
    int* s_misc = (int*)(s_red + kW12 * 4 + 8);
    uint32_t* s_hist = (uint32_t*)(s_misc + 16);                       // pass 1 with p.hist: [2][kTopkBins] counts of the final scores
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x % p.Hkv;
    const int rest = blockIdx.x / p.Hkv;
    const int b = rest / p.S, sp = rest % p.S;
    const int bg = b * p.Hkv + g;
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * CB;
    float* out_k = p.ans_k + (int64_t)bg * p.N;
    float* out_v = p.ans_v + (int64_t)bg * p.N;
    const bool count_scores = PASS == 1 && p.hist != nullptr;

    s_mk[tid] = 0u;
    if (count_scores)
        for (int i = tid; i < 2 * kTopkBins; i += kT12) s_hist[i] = 0u;
    if (wave < 2) {
        const int r = lower_bound64(idx_k, p.k_k, (int)(wave ? t1 : t0), lane);
        if (lane == 0) s_misc[wave] = r;
    }
    __syncthreads();
    for (int i = s_misc[0] + tid; i < s_misc[1]; i += kT12) {
        const int rel = idx_k[i] - (int)t0;
        atomicOr(&s_mk[rel >> 5], 1u << (rel & 31));
    }

    const int n_walks = (p.G + NHA - 1) / NHA;
#pragma unroll 1
    for (int hh = 0; hh < n_walks; ++hh) {
        const int hfirst = g * p.G + NHA * hh;                         // first query head of this walk
        const int nh = (p.G - NHA * hh) < NHA ? (p.G - NHA * hh) : NHA;
        __syncthreads();                                               // the previous walk no longer reads the table or s_red
        if (tid < 2 * kD) s_qf[tid] = ((tid >> 7) < nh) ? (float)p.q[((int64_t)b * p.Hq + hfirst) * kD + tid] : 0.f;
        {
            const float4_t* tb = p.tab + (int64_t)bg * kM12 * kC12;
#pragma unroll 4
            for (int e = tid; e < kM12 * kC12; e += kT12) {
                const float4_t t = tb[e];
                if constexpr (NHA == 2) s_lut[e] = hh ? float2{t[2], t[3]} : float2{t[0], t[1]};
                else s_lut[e] = hh == 0 ? t[0] : (hh == 1 ? t[1] : (hh == 2 ? t[2] : t[3]));
            }
        }
        __syncthreads();
        if (wave < 2) {                                                // ||q_h||_2
            const float a = s_qf[wave * kD + lane], c = s_qf[wave * kD + 64 + lane];
            const float ss = wave_sum(fmaf(a, a, c * c));
            if (lane == 0) s_red[kW12 * 4 + wave] = sqrtf(ss);
        }
        if (PASS == 1 && (wave == 2 || wave == 3)) {                   // log-sum-exp from the S partials of pass 0: a wave per head
            const int h = wave - 2;
            float v = 0.f;
            if (h < nh) {
                const float2* sp_ = (const float2*)(p.stat_part + ((int64_t)b * p.Hq + hfirst + h) * p.S * 2);
                float m = kNegBig, l = 0.f;                            // per-lane (reference, sum) over its share of the pairs
                for (int s = lane; s < p.S; s += 64) {
                    const float2 ml = sp_[s];
                    const float mn = fmaxf(m, ml.x);
                    l = l * exp2f(m - mn) + ml.y * exp2f(ml.x - mn);
                    m = mn;
                }
                const float mw = wave_max(m);
                l = wave_sum(l * exp2f(m - mw));
                v = mw + log2f(l);
            }
            if (lane == 0) s_red[kW12 * 4 + 4 + h] = v;
        }
        __syncthreads();
        const float qn0 = s_red[kW12 * 4], qn1 = s_red[kW12 * 4 + 1];
        const float lse0 = s_red[kW12 * 4 + 4], lse1 = s_red[kW12 * 4 + 5];
        float m_run[2] = {kNegBig, kNegBig}, l_run[2] = {0.f, 0.f};

        auto consume = [&](float s0, float s1, int64_t tok) {
            if (PASS == 0) {
                const float sv[2] = {s0, s1};
#pragma unroll
                for (int h = 0; h < NHA; ++h) {
                    const float x = sv[h] - m_run[h];
                    if (x > 64.f) {                                    // first token (reference = kNegBig) or a big jump
                        l_run[h] = l_run[h] * fast_exp2(-x) + 1.f;
                        m_run[h] = sv[h];
                    } else {
                        l_run[h] += fast_exp2(x);
                    }
                }
            } else {
                const float a0 = fast_exp2(s0 - lse0);
                const float a1 = (NHA > 1 && nh > 1) ? fast_exp2(s1 - lse1) : 0.f;
                const float t0_ = a0 * qn0, t1_ = a1 * qn1;
                float av = a0 + a1;
                float ak = fmaf(-a0, t0_, t0_) + fmaf(-a1, t1_, t1_);
                if (hh > 0) { av += out_v[tok]; ak += out_k[tok]; }    // earlier walks' heads, written by this thread
                out_v[tok] = av;
                out_k[tok] = ak;
                if (count_scores && hh == n_walks - 1) {               // final values: the selection that follows starts from these counts
                    atomicAdd(&s_hist[float_key(ak) >> 21], 1u);
                    atomicAdd(&s_hist[kTopkBins + (float_key(av) >> 21)], 1u);
                }
            }
        };

        // ---- stream: one token per lane, code loads one round ahead; K-anchored tokens are left to the loop below
        uint32_t nw[3] = {0u, 0u, 0u};
        if (t0 + tid < t1) load_cw<kD12>(ck, t0 + tid, nw);
        for (int64_t tok = t0 + tid; tok < t1; tok += kT12) {
            const uint32_t kw[3] = {nw[0], nw[1], nw[2]};
            if (tok + kT12 < t1) load_cw<kD12>(ck, tok + kT12, nw);
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int m = 0; m < kM12; ++m) {
                const lut_t e = s_lut[m * kC12 + code12(kw, m)];
                if constexpr (NHA == 2) { s0 += e.x; s1 += e.y; }
                else s0 += e;
            }
            const int rel = (int)(tok - t0);
            if (!((s_mk[rel >> 5] >> (rel & 31)) & 1u)) consume(s0, s1, tok);
        }
        // ---- K-anchored tokens: score from the FP16 row, 16 lanes per token and 8 channels each; blocks of 64 list
        // entries are dealt round-robin over the S workgroups of the head
        {
            const int sub = lane >> 4, l16 = lane & 15;
            float qv[NHA][8];
#pragma unroll
            for (int h = 0; h < NHA; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) qv[h][e] = s_qf[h * kD + 8 * l16 + e];
            for (int i0 = sp * (4 * kW12) + 4 * wave; i0 < p.k_k; i0 += p.S * (4 * kW12)) {
                const int i = i0 + sub;
                const bool on = i < p.k_k;
                const int64_t tok = on ? idx_k[i] : t0;
                const half8_t v = *(const half8_t*)(p.rows_k + ((int64_t)bg * p.k_k + (on ? i : 0)) * kD + 8 * l16);
                float s[2] = {0.f, 0.f};
#pragma unroll
                for (int h = 0; h < NHA; ++h) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) d = fmaf(qv[h][e], (float)v[e], d);
#pragma unroll
                    for (int off = 1; off < 16; off <<= 1) d += __shfl_xor(d, off, 64);
                    s[h] = d * p.c1;
                }
                if (on && l16 == 0) consume(s[0], s[1], tok);
            }
        }
        if (PASS == 0) {
#pragma unroll
            for (int h = 0; h < NHA; ++h) {
                const float m_w = wave_max(m_run[h]);
                const float l_w = wave_sum(l_run[h] * fast_exp2(m_run[h] - m_w));
                if (lane == 0) { s_red[wave * 4 + h] = m_w; s_red[wave * 4 + 2 + h] = l_w; }
            }
            __syncthreads();
            if (tid < nh) {
                float m = kNegBig;
                for (int w = 0; w < kW12; ++w) m = fmaxf(m, s_red[w * 4 + tid]);
                float l = 0.f;
                for (int w = 0; w < kW12; ++w) l += s_red[w * 4 + 2 + tid] * fast_exp2(s_red[w * 4 + tid] - m);
                float* dst = p.stat_part + (((int64_t)b * p.Hq + hfirst + tid) * p.S + sp) * 2;
                dst[0] = m;
                dst[1] = l;
            }
        }
    }
    if (count_scores) {
        __syncthreads();
        const int64_t n_bg = (int64_t)gridDim.x / p.S;                 // B * Hkv: the V rows follow the K rows
        uint32_t* hk = p.hist + (int64_t)bg * 2 * kTopkBins;
        uint32_t* hv = p.hist + (n_bg + bg) * 2 * kTopkBins;
        for (int i = tid; i < kTopkBins; i += kT12) {
            if (s_hist[i]) atomicAdd(&hk[i], s_hist[i]);
            if (s_hist[kTopkBins + i]) atomicAdd(&hv[i], s_hist[kTopkBins + i]);
        }
    }
}

struct D12Plan {
    int S, chunk;
    size_t off_part, off_tab, off_amax, off_stat, off_early, total;
};

D12Plan d12_plan(const Geom& g, int64_t N)
{
    D12Plan pl;
    const int64_t bgc = (int64_t)g.B * g.Hkv;
    int64_t S = (256 + bgc - 1) / bgc;                                 // about one workgroup per CU
    const int64_t s_max = (N + 1023) / 1024;
    if (S > s_max) S = s_max;
    if (S < 1) S = 1;
    int64_t chunk = ((N + S - 1) / S + 63) / 64 * 64;
    if (chunk > kChunkMax) chunk = kChunkMax;
    if (chunk < 64) chunk = 64;
    S = (N + chunk - 1) / chunk;
    if (S < 1) S = 1;
    pl.S = (int)S;
    pl.chunk = (int)chunk;
    size_t off = 0;
    pl.off_part = off; off += align_up((size_t)g.B * g.Hq * S * (kD + 2) * sizeof(float));
    pl.off_tab = off;  off += align_up((size_t)g.B * g.Hkv * g.M * kC12 * sizeof(float4_t));
    pl.off_amax = off; off += align_up((size_t)g.B * g.Hkv * tab_blocks(g.d) * kNH * sizeof(float));
    pl.off_stat = off; off += align_up((size_t)g.B * g.Hq * S * 2 * sizeof(float));
    pl.off_early = off;                                                // first-walk scores: only where a table holds fewer heads than the group has
    if (g.G > heads_per_table(g.d)) off += align_up((size_t)g.B * g.Hkv * N * sizeof(float2));
    pl.total = off;
    return pl;
}

template <int DS>
hipError_t launch_decode12_t(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st)
{
    const D12Plan pl = d12_plan(g, a.N);
    constexpr size_t lds = d12_lds(DS);
    static const hipError_t setup = []() {
        const hipError_t e1 = hipFuncSetAttribute((const void*)decode12_kernel<DS, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e1 != hipSuccess) return e1;
        return hipFuncSetAttribute((const void*)decode12_kernel<DS, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    }();
    if (setup != hipSuccess) return setup;
    if ((int64_t)g.B * g.Hkv * pl.S > 0x7fffffffLL) return hipErrorInvalidValue;
    if ((int64_t)g.B * g.Hkv * a.k_v * kD * 2 >= 0x7fffffffLL) return hipErrorInvalidValue;   // 31-bit byte offsets into rows_v
    D12Params p;
    p.q = a.q; p.codes_k = a.codes_k; p.codes_v = a.codes_v; p.cb_k = a.cb_k; p.cb_v = a.cb_v;
    p.idx_k = a.idx_k; p.idx_v = a.idx_v; p.rows_k = a.rows_k; p.rows_v = a.rows_v;
    char* w = (char*)ws;
    p.part = (float*)(w + pl.off_part); p.tab = (const float4_t*)(w + pl.off_tab); p.tab_amax = (const float*)(w + pl.off_amax);
    p.N = a.N; p.N_cap = a.N_cap; p.k_k = (int)a.k_k; p.k_v = (int)a.k_v;
    p.c1 = a.scale * kLog2e; p.Hq = g.Hq; p.Hkv = g.Hkv; p.G = g.G; p.S = a.N > 0 ? pl.S : 0; p.chunk = pl.chunk;
    p.early = (float2*)(w + pl.off_early);
    p.given = (const float4_t*)a.given_scores;
    if (a.given_scores && (a.k_k != 0 || a.ans_k || a.ans_v)) return hipErrorInvalidValue;     // the scores cover the K anchors already
    if (a.N > 0 && a.given_scores) {
        hipLaunchKernelGGL((decode12_kernel<DS, true>), dim3((unsigned)(g.B * g.Hkv * pl.S)), dim3(kT12), lds, st, p);
    } else if (a.N > 0) {
        hipLaunchKernelGGL(d12_table_kernel<DS>, dim3((unsigned)(g.B * g.Hkv), tab_blocks(DS)), dim3(kTabThreads), 0, st, a.q,
                           a.cb_k, p.c1, g.Hq, g.Hkv, g.G, (float4_t*)(w + pl.off_tab), (float*)(w + pl.off_amax));
        hipLaunchKernelGGL((decode12_kernel<DS, false>), dim3((unsigned)(g.B * g.Hkv * pl.S)), dim3(kT12), lds, st, p);
    }
    hipLaunchKernelGGL(decode12_merge, dim3((unsigned)(g.B * g.Hq)), dim3(kD), 0, st, (const float*)p.part, p.S, a.out);
    if (a.ans_k && a.N > 0) {
        static const hipError_t setup_ans = []() {
            hipError_t e1 = hipFuncSetAttribute((const void*)d12_ans_kernel<DS, 0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)kD12AnsLds);
            if (e1 != hipSuccess) return e1;
            return hipFuncSetAttribute((const void*)d12_ans_kernel<DS, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kD12AnsLds);
        }();
        if (setup_ans != hipSuccess) return setup_ans;
        D12AnsParams d;
        d.q = a.q; d.codes_k = a.codes_k; d.idx_k = a.idx_k; d.rows_k = a.rows_k; d.tab = p.tab;
        d.stat_part = (float*)(w + pl.off_stat); d.ans_k = a.ans_k; d.ans_v = a.ans_v; d.N = a.N; d.N_cap = a.N_cap;
        d.k_k = (int)a.k_k; d.c1 = p.c1; d.Hq = g.Hq; d.Hkv = g.Hkv; d.G = g.G; d.S = pl.S; d.chunk = pl.chunk;
        d.hist = a.topk_hist;
        const unsigned grid = (unsigned)(g.B * g.Hkv * pl.S);
        hipLaunchKernelGGL((d12_ans_kernel<DS, 0>), dim3(grid), dim3(kT12), kD12AnsLds, st, d);
        hipLaunchKernelGGL((d12_ans_kernel<DS, 1>), dim3(grid), dim3(kT12), kD12AnsLds, st, d);
    }
    return hipGetLastError();
}

}  // namespace

size_t decode12_workspace_bytes(const Geom& g, int64_t N) { return d12_plan(g, N).total; }

hipError_t launch_decode12(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st)
{
    return g.d == 32 ? launch_decode12_t<32>(g, a, ws, st) : launch_decode12_t<16>(g, a, ws, st);
}

}  // namespace antkv
