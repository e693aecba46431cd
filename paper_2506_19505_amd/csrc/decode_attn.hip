// Decode attention over VQ codes + FP16 anchor tokens (paper Sec. 2.1 Attn with one query row; Sec. 3,
// Fig. 2(b): anchor tokens stay FP16, every other token is read from its codes), and the decode-time
// Anchor Score (Sec. 3.2 last paragraph: Eq. (4) evaluated for the single decode query).
//
// One launch holds two kinds of workgroups (8 waves each):
//
//  * stream workgroups own a contiguous token range of one (sequence, KV head).  They build the
//    q.centroid lookup table LUT[m][c][head] (16-bit fixed point, pre-multiplied by scale*log2e) and copy the V
//    codebook into LDS once, then every wave walks over 64-token tiles:
//      K side  one lane per token: 16-byte coalesced code loads, one 8-byte LUT gather per sub-space
//              serves the group's four query heads, exact integer accumulation;
//      softmax base-2 online softmax against a lazily updated reference maximum (the wave only pays
//              the cross-lane reduction when some score exceeds the reference);
//      V side  P (fp16) goes through a 512-byte LDS staging buffer into MFMA A-operand layout; V
//              centroids are fetched from the LDS codebook with ds_read_b64_tr_b16, whose lane
//              transposition yields the MFMA B operand (tokens along k) directly;
//              v_mfma_f32_16x16x32_f16 accumulates P.V in fp32.
//    Tokens that have an FP16 anchor row (for K or for V) are masked out of the stream via an LDS bitmap.
//
//  * anchor workgroups take 32-token tiles of the anchor lists (balanced by list index, not by position):
//    they stage K_eff / V_eff rows (the FP16 row, or the de-quantised codes when only the other tensor
//    of that token is anchored) in LDS and run the same two MFMA contractions on dense rows.
//
// Every workgroup writes one partial (reference max, sum, accumulator) per query head; a second kernel
// merges the partials by log-sum-exp and rounds once to fp16.
#include "common.h"

namespace antkv {

namespace {

constexpr int kDaWaves = 8;
constexpr int kDaThreads = kDaWaves * 64;
constexpr int kNH = 4;                 // query-head slots per workgroup (group size G <= 4)
constexpr float kPShift = 8.0f;        // P is scaled by 2^8 so that small weights stay normal in fp16
constexpr float kEmptyRef = -1.0e4f;   // softmax reference before any token was seen: finite, below every real score,
                                       // and far above the masked score kNegBig so that exp2(masked - ref) is 0
constexpr int kAnchorTilesPerWave = 1;
constexpr int kAnchorTilesPerWg = kDaWaves * kAnchorTilesPerWave;

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) short4_t lds_short4;

__device__ __forceinline__ half4_t lds_read_tr16(const lds_char* base, uint32_t off)
{
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(base + off));
    return __builtin_bit_cast(half4_t, v);
}

template <int SRC>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, SRC * 0x55, 0xf, 0xf, true);
}

// max over the 64 lanes, result uniform
__device__ __forceinline__ float wave_max_uniform(float v)
{
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true)));   // quad_perm [1,0,3,2]
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true)));   // quad_perm [2,3,0,1]
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true)));  // row_half_mirror
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true)));  // row_mirror
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// sum over each row of 16 lanes, result in all 16 lanes
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true));
    return v;
}

// first index in arr[0..n) whose value is >= key; executed by a whole wave, result uniform
__device__ int wave_lower_bound(const int32_t* __restrict__ arr, int n, int key, int lane)
{
    int lo = 0, hi = n;
    while (hi > lo) {
        const int span = hi - lo;
        const int step = (span + 63) >> 6;
        const int p = lo + lane * step;
        const int v = (p < hi) ? arr[p] : 0x7fffffff;
        const int c = __builtin_popcountll(__ballot(v < key));   // probes 0..c-1 are below the key
        if (c == 0) { hi = lo; break; }
        const int nlo = lo + (c - 1) * step + 1;
        const int nhi = lo + c * step;
        lo = nlo;
        hi = nhi < hi ? nhi : hi;
        if (step == 1) { lo = hi = nlo; break; }
    }
    return lo;
}

// per-lane binary search: position of key in sorted arr[0..n) or -1
__device__ __forceinline__ int find_sorted(const int32_t* __restrict__ arr, int n, int key)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (arr[mid] < key) lo = mid + 1; else hi = mid;
    }
    return (lo < n && arr[lo] == key) ? lo : -1;
}

struct DaParams {
    const half_t* q;
    const uint8_t *codes_k, *codes_v;
    const half_t *cb_k, *cb_v;
    const int32_t *idx_k, *idx_v;
    const half_t *rows_k, *rows_v;
    float* part;                // [B][Hq][slots][kD + 2]
    int64_t N, N_cap;
    int k_k, k_v;
    float c1;                   // scale * log2(e)
    int Hq, Hkv, G;
    int S;                      // stream splits per (b, g)
    int A;                      // anchor workgroups per (b, g)
    int64_t chunk;              // tokens per stream split (multiple of 64)
};

// LDS layout (bytes).  The stream layout and the anchor layout overlap; a workgroup uses one of them.
template <int DSUB>
struct Lds {
    static constexpr int M = kD / DSUB;
    static constexpr int lut = 0;                                  // [M][256][4] int16
    static constexpr int cbv = lut + M * 256 * 8;                  // [M][256][DSUB] fp16 = 64 KB
    static constexpr int pst = cbv + 65536;                        // [waves][4][64] fp16
    static constexpr int qf = pst + kDaWaves * 512;                // [4][128] fp32
    static constexpr int red = qf + 2048;                          // [waves][8] fp32 + misc ints
    static constexpr int mask = red + kDaWaves * 32 + 64;          // bitmap over the token range
    static constexpr int mask_words = 1024;                        // up to 32768 tokens per split
    static constexpr int stream_total = mask + mask_words * 4;
    // anchor layout: per wave a 32 x 128 fp16 row tile (8 KB) + P staging + slot table
    static constexpr int a_rows = 0;                               // [waves][32][128] fp16
    static constexpr int a_pst = a_rows + kDaWaves * 8192;         // [waves][4][32] fp16
    static constexpr int a_qf = a_pst + kDaWaves * 256;
    static constexpr int a_red = a_qf + 2048;
    static constexpr int anchor_total = a_red + kDaWaves * 32 + 64;
    static constexpr int total = stream_total > anchor_total ? stream_total : anchor_total;
    // merge buffer re-uses the front of LDS after the main loop: [waves][4][128] fp32 = 32 KB
    static constexpr int mrg = 0;
};

// Merge the 16 waves' (m_ref, l, acc) into one partial and write it.  acc is in MFMA C layout:
// lanes 0..15 of a wave hold, for slab c and register r, head r and channel 16c + lane.
template <int DSUB>
__device__ void wg_merge_and_store(char* smem, float (&m_ref)[kNH], float (&l_sum)[kNH], float4_t (&acc)[8],
                                   float* __restrict__ part_bg, int slot, int slots, int nheads, int red_off)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* s_red = (float*)(smem + red_off);
    __syncthreads();   // everyone is done with the tables in LDS
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < kNH; ++h) { s_red[wave * 8 + h] = m_ref[h]; s_red[wave * 8 + 4 + h] = l_sum[h]; }
    }
    __syncthreads();
    float m_all[kNH], l_all[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) {
        float m = kNegBig;
        for (int w = 0; w < kDaWaves; ++w) m = fmaxf(m, s_red[w * 8 + h]);
        float l = 0.f;
        for (int w = 0; w < kDaWaves; ++w) l += s_red[w * 8 + 4 + h] * fast_exp2(s_red[w * 8 + h] - m);
        m_all[h] = m;
        l_all[h] = l;
    }
    float* s_mrg = (float*)(smem + Lds<DSUB>::mrg);
    if (lane < 16) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int r = 0; r < kNH; ++r)
                s_mrg[(wave * kNH + r) * kD + 16 * c + lane] = acc[c][r] * fast_exp2(m_ref[r] - m_all[r]);
    }
    __syncthreads();
    if (tid < kNH * kD) {
        const int h = tid >> 7, dim = tid & 127;
        if (h < nheads) {
            float s = 0.f;
            for (int w = 0; w < kDaWaves; ++w) s += s_mrg[(w * kNH + h) * kD + dim];
            float* dst = part_bg + ((int64_t)h * slots + slot) * (kD + 2);
            dst[dim] = s;
            if (dim == 0) { dst[kD] = m_all[h]; dst[kD + 1] = l_all[h]; }
        }
    }
}

template <int DSUB>
__global__ __launch_bounds__(kDaThreads) void decode_attn_kernel(const DaParams p)
{
    constexpr int M = kD / DSUB;
    constexpr int CW = M / 4;              // code dwords per token
    using L = Lds<DSUB>;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    const lds_char* lsm = (const lds_char*)smem_u4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per_bg = p.A + p.S;
    const int bg = blockIdx.x / per_bg, role = blockIdx.x % per_bg;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int nheads = p.G;               // <= kNH
    const int h0 = g * p.G;
    const int slots = per_bg;
    float* part_bg = p.part + ((int64_t)b * p.Hq + h0) * slots * (kD + 2);
    const half_t* qb = p.q + ((int64_t)b * p.Hq + h0) * kD;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const int32_t* idx_v = p.idx_v + (int64_t)bg * p.k_v;

    float m_ref[kNH], l_lane[kNH];
    float4_t acc[8];
#pragma unroll
    for (int h = 0; h < kNH; ++h) { m_ref[h] = kEmptyRef; l_lane[h] = 0.f; }
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};

    // MFMA lane coordinates
    const int kgrp = lane >> 4;           // tr block / k group
    const int tj = (lane >> 2) & 3;       // token within a group of four
    const int tq = lane & 3;              // 8-byte chunk of a 32-byte channel slab / quad lane
    const int arow = lane & 15;           // A-operand row (head) / C column (channel)

    if (role >= p.A) {
        // ======================================================================= stream role
        const int sp = role - p.A;
        const int64_t t0 = (int64_t)sp * p.chunk;
        const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
        float* s_qf = (float*)(smem + L::qf);
        int* s_misc = (int*)(smem + L::red + kDaWaves * 32);
        uint32_t* s_mask = (uint32_t*)(smem + L::mask);

        if (tid < kNH * kD) {
            const int h = tid >> 7;
            s_qf[tid] = (h < nheads) ? (float)qb[tid] : 0.f;
        }
        for (int i = tid; i < L::mask_words; i += kDaThreads) s_mask[i] = 0u;
        {   // V codebook -> LDS
            const uint4_t* src = (const uint4_t*)(p.cb_v + (size_t)g * 32768);
            uint4_t* dst = (uint4_t*)(smem + L::cbv);
            for (int i = tid; i < 4096; i += kDaThreads) dst[i] = src[i];
        }
        // anchor list ranges that fall into [t0, t1)
        if (wave < 4) {
            const int32_t* arr = (wave < 2) ? idx_k : idx_v;
            const int n = (wave < 2) ? p.k_k : p.k_v;
            const int64_t key = (wave & 1) ? t1 : t0;
            const int r = wave_lower_bound(arr, n, (int)key, lane);
            if (lane == 0) s_misc[wave] = r;
        }
        __syncthreads();
        // LUT[m][c][h] = c1 * q_h[m*d : (m+1)*d] . cb_k[g][m][c], stored as 16-bit fixed point with one scale per
        // head (quantum = max|LUT_h| / 32767): the per-token sum over sub-spaces is then exact integer arithmetic
        // and the table error is uniform instead of growing with the entry's magnitude as it would in fp16.
        float lut_q[kNH];
        {
            const half_t* cbk = p.cb_k + (size_t)g * 32768;
            // one table entry (4 heads) in fp32; evaluated twice (range pass, quantise pass) to keep registers low
            auto entry = [&](int e, float (&val)[kNH]) {
                const int m = e >> 8;
                float cen[DSUB];
                if (DSUB == 4) {
                    const half4_t v = *(const half4_t*)(cbk + e * 4);
#pragma unroll
                    for (int t = 0; t < 4; ++t) cen[t] = (float)v[t];
                } else {
#pragma unroll
                    for (int u = 0; u < DSUB / 8; ++u) {
                        const half8_t v = *(const half8_t*)(cbk + e * DSUB + 8 * u);
#pragma unroll
                        for (int t = 0; t < 8; ++t) cen[8 * u + t] = (float)v[t];
                    }
                }
#pragma unroll
                for (int h = 0; h < kNH; ++h) {
                    float sdot = 0.f;
#pragma unroll
                    for (int t = 0; t < DSUB; ++t) sdot = fmaf(s_qf[h * kD + m * DSUB + t], cen[t], sdot);
                    val[h] = sdot * p.c1;
                }
            };
            float amax[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
            for (int e = tid; e < M * 256; e += kDaThreads) {
                float val[kNH];
                entry(e, val);
#pragma unroll
                for (int h = 0; h < kNH; ++h) amax[h] = fmaxf(amax[h], fabsf(val[h]));
            }
            float* s_red = (float*)(smem + L::red);
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float wm = wave_max_uniform(amax[h]);
                if (lane == 0) s_red[wave * 8 + h] = wm;
            }
            __syncthreads();
            float inv_q[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                float r = 0.f;
                for (int wv = 0; wv < kDaWaves; ++wv) r = fmaxf(r, s_red[wv * 8 + h]);
                lut_q[h] = (r > 0.f) ? r / 32767.0f : 1.0f;
                inv_q[h] = (r > 0.f) ? 32767.0f / r : 0.f;
            }
            uint2_t* s_lut = (uint2_t*)(smem + L::lut);
#pragma unroll 1
            for (int e = tid; e < M * 256; e += kDaThreads) {
                float val[kNH];
                entry(e, val);
                int qv[kNH];
#pragma unroll
                for (int h = 0; h < kNH; ++h) qv[h] = (int)rintf(val[h] * inv_q[h]);
                s_lut[e] = uint2_t{((uint32_t)qv[0] & 0xffffu) | ((uint32_t)qv[1] << 16),
                                   ((uint32_t)qv[2] & 0xffffu) | ((uint32_t)qv[3] << 16)};
            }
            // bitmap of anchored tokens in this range
            const int lo_k = s_misc[0], hi_k = s_misc[1], lo_v = s_misc[2], hi_v = s_misc[3];
            for (int i = lo_k + tid; i < hi_k; i += kDaThreads) {
                const int rel = idx_k[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
            for (int i = lo_v + tid; i < hi_v; i += kDaThreads) {
                const int rel = idx_v[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        __syncthreads();

        // lane -> token position inside a 64-token tile, chosen so that the four lanes of a quad hold
        // the V codes of exactly the four tokens whose centroids that quad must fetch for the MFMA
        const int pos = 32 * (tq >> 1) + 8 * kgrp + 4 * (tq & 1) + tj;
        half_t* s_p = (half_t*)(smem + L::pst) + wave * 256;          // [4][64]
        const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * M;
        const uint8_t* cv = p.codes_v + (int64_t)bg * p.N_cap * M;
        // V gather address pieces (bytes): ((m*256 + code)*DSUB + within)*2
        uint32_t v_lane_off, v_shift_lane;
        if (DSUB == 8) { v_lane_off = (tq >> 1) * 4096 + (tq & 1) * 8; v_shift_lane = 8 * (tq >> 1); }
        else if (DSUB == 4) { v_lane_off = tq * 2048; v_shift_lane = 8 * tq; }
        else { v_lane_off = tq * 8; v_shift_lane = 0; }
        v_lane_off += L::cbv;

        const int64_t n_tiles = (t1 - t0 + 63) >> 6;
        for (int64_t tile = wave; tile < n_tiles; tile += kDaWaves) {
            const int64_t tok = t0 + tile * 64 + pos;
            const bool in_range = tok < t1;
            const int64_t ltok = in_range ? tok : (p.N - 1);
            uint32_t kw[CW], vw[CW];
            if (CW == 2) {
                const uint2_t a = *(const uint2_t*)(ck + ltok * M), c = *(const uint2_t*)(cv + ltok * M);
                kw[0] = a[0]; kw[1] = a[1]; vw[0] = c[0]; vw[1] = c[1];
            } else {
#pragma unroll
                for (int i = 0; i < CW / 4; ++i) {
                    const uint4_t a = *(const uint4_t*)(ck + ltok * M + 16 * i), c = *(const uint4_t*)(cv + ltok * M + 16 * i);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { kw[4 * i + e] = a[e]; vw[4 * i + e] = c[e]; }
                }
            }
            const int rel = (int)(tok - t0);
            const bool masked = !in_range || ((s_mask[(rel >> 5) & (L::mask_words - 1)] >> (rel & 31)) & 1u);

            // ---- K side: scores in log2 units
            int si[kNH] = {0, 0, 0, 0};
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const uint32_t code = (kw[m >> 2] >> (8 * (m & 3))) & 255u;
                const uint2_t e = *(const uint2_t*)(smem + L::lut + (m * 256 + code) * 8);
                // plain integer half-word adds (the sdot2 builtin mis-compiles here: it drops the second dword)
                si[0] += (int)(short)(e[0] & 0xffffu);
                si[1] += ((int)e[0]) >> 16;
                si[2] += (int)(short)(e[1] & 0xffffu);
                si[3] += ((int)e[1]) >> 16;
            }
            float s[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) s[h] = (float)si[h] * lut_q[h];
            bool grow = false;
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                s[h] = masked ? kNegBig : s[h];
                grow = grow || (s[h] > m_ref[h] + kPShift);
            }
            if (__any(grow)) {   // some score exceeds the running maximum: move the reference, rescale
#pragma unroll
                for (int h = 0; h < kNH; ++h) {
                    const float mx = wave_max_uniform(s[h]);
                    const float m_new = fmaxf(m_ref[h], mx - kPShift);
                    const float alpha = fast_exp2(m_ref[h] - m_new);
                    l_lane[h] *= alpha;
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[c][h] *= alpha;
                    m_ref[h] = m_new;
                }
            }
            float pw[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                pw[h] = fast_exp2(s[h] - m_ref[h]);
                l_lane[h] += pw[h];
                s_p[h * 64 + pos] = (half_t)pw[h];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();

            // ---- V side
            // V codes of the quad's four tokens: quad lane 2u+hi holds token (u, hi)
            uint32_t vq[4][CW];
#pragma unroll
            for (int i = 0; i < CW; ++i) {
                vq[0][i] = quad_bcast<0>(vw[i]);
                vq[1][i] = quad_bcast<1>(vw[i]);
                vq[2][i] = quad_bcast<2>(vw[i]);
                vq[3][i] = quad_bcast<3>(vw[i]);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                half8_t pa = *(const half8_t*)(s_p + (arow & 3) * 64 + 32 * u + 8 * kgrp);
                if (arow >= kNH) pa = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    half4_t vb[2];
#pragma unroll
                    for (int hi = 0; hi < 2; ++hi) {
                        // channel slab c (16 channels), this lane's chunk tq: sub-space and code byte
                        int dw, sh_c, moff;
                        if (DSUB == 8) { dw = c >> 1; sh_c = 16 * (c & 1); moff = c * 8192; }
                        else if (DSUB == 4) { dw = c; sh_c = 0; moff = c * 8192; }
                        else { dw = c >> 2; sh_c = 8 * (c & 3); moff = c * 8192; }
                        const uint32_t code = (vq[2 * u + hi][dw] >> (sh_c + v_shift_lane)) & 255u;
                        vb[hi] = lds_read_tr16(lsm, code * (2 * DSUB) + v_lane_off + moff);
                    }
                    const half8_t bop = {vb[0][0], vb[0][1], vb[0][2], vb[0][3], vb[1][0], vb[1][1], vb[1][2], vb[1][3]};
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, bop, acc[c], 0, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        float l_sum[kNH];
#pragma unroll
        for (int h = 0; h < kNH; ++h) l_sum[h] = wave_sum(l_lane[h]);
        wg_merge_and_store<DSUB>(smem, m_ref, l_sum, acc, part_bg, p.A + sp, slots, nheads, L::red);
        return;
    }

    // =========================================================================== anchor role
    {
        const int aw = role;                                  // anchor workgroup index within (b, g)
        const int n_items = p.k_k + p.k_v;                    // K-anchor entries, then V-anchor entries
        float* s_qf = (float*)(smem + L::a_qf);
        if (tid < kNH * kD) {
            const int h = tid >> 7;
            s_qf[tid] = (h < nheads) ? (float)qb[tid] : 0.f;
        }
        __syncthreads();
        // Q as MFMA A operand: row = head, 4 k-steps of 32 channels
        half8_t qa[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                qa[st][e] = (arow < nheads) ? qb[arow * kD + 32 * st + 8 * kgrp + e] : (half_t)0.f;
        }
        half_t* s_rows = (half_t*)(smem + L::a_rows) + wave * 4096;     // [32][128]
        half_t* s_p = (half_t*)(smem + L::a_pst) + wave * 128;          // [4][32]
        const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * M;
        const uint8_t* cv = p.codes_v + (int64_t)bg * p.N_cap * M;
        const half_t* cbk = p.cb_k + (size_t)g * 32768;
        const half_t* cbv = p.cb_v + (size_t)g * 32768;

        for (int tw = 0; tw < kAnchorTilesPerWave; ++tw) {
            const int tile = (aw * kDaWaves + wave) * kAnchorTilesPerWave + tw;
            const int item0 = tile * 32;
            if (item0 >= n_items) break;
            // lanes 0..31 each own one item of the tile: resolve where its K and V rows come from
            int my_tok = -1, my_kslot = -1, my_vslot = -1;     // slot >= 0: FP16 row; -1: from codes
            bool my_valid = false;
            if (lane < 32) {
                const int it = item0 + lane;
                if (it < p.k_k) {
                    my_tok = idx_k[it];
                    my_kslot = it;
                    my_vslot = find_sorted(idx_v, p.k_v, my_tok);
                    my_valid = true;
                } else if (it < n_items) {
                    my_tok = idx_v[it - p.k_k];
                    my_vslot = it - p.k_k;
                    my_valid = find_sorted(idx_k, p.k_k, my_tok) < 0;   // handled as a K item otherwise
                }
            }
            // ---- stage K_eff rows: half-wave hw fills rows hw, hw+2, ...; lane covers 4 channels
            const int hw = lane >> 5, l32 = lane & 31;
            for (int r = hw; r < 32; r += 2) {
                const int tok = __shfl(my_tok, r, 64);
                const int kslot = __shfl(my_kslot, r, 64);
                const bool valid = __shfl((int)my_valid, r, 64) != 0;
                half4_t v = {0, 0, 0, 0};
                if (valid) {
                    if (kslot >= 0) {
                        v = *(const half4_t*)(p.rows_k + ((int64_t)bg * p.k_k + kslot) * kD + 4 * l32);
                    } else {
                        const int dim = 4 * l32, m = dim / DSUB;
                        const int code = ck[(int64_t)tok * M + m];
                        v = *(const half4_t*)(cbk + (m * 256 + code) * DSUB + (dim % DSUB));
                    }
                }
                *(half4_t*)(s_rows + r * kD + 4 * l32) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // ---- scores: S[head][item] for the two 16-item halves
            float sc[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float4_t c4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const half8_t kb = *(const half8_t*)(s_rows + (16 * u + arow) * kD + 32 * st + 8 * kgrp);
                    c4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[st], kb, c4, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[u][r] = c4[r] * p.c1;   // lanes 0..15: head r, item 16u + lane
            }
            // validity of item 16u + arow, then the tile maximum per head
            float mx[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) mx[h] = kNegBig;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bool valid = __shfl((int)my_valid, 16 * u + arow, 64) != 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (!(valid && kgrp == 0)) sc[u][r] = kNegBig;
                    mx[r] = fmaxf(mx[r], sc[u][r]);
                }
            }
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float m_tile = wave_max_uniform(mx[h]);
                const float m_new = fmaxf(m_ref[h], m_tile - kPShift);
                const float alpha = fast_exp2(m_ref[h] - m_new);
                l_lane[h] *= alpha;
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c][h] *= alpha;
                m_ref[h] = m_new;
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pw = fast_exp2(sc[u][r] - m_ref[r]);       // 0 for masked / non-row lanes
                    l_lane[r] += pw;
                    if (kgrp == 0) s_p[r * 32 + 16 * u + arow] = (half_t)pw;
                }
            __builtin_amdgcn_wave_barrier();
            // ---- stage V_eff rows over the K rows
            for (int r = hw; r < 32; r += 2) {
                const int tok = __shfl(my_tok, r, 64);
                const int vslot = __shfl(my_vslot, r, 64);
                const bool valid = __shfl((int)my_valid, r, 64) != 0;
                half4_t v = {0, 0, 0, 0};
                if (valid) {
                    if (vslot >= 0) {
                        v = *(const half4_t*)(p.rows_v + ((int64_t)bg * p.k_v + vslot) * kD + 4 * l32);
                    } else {
                        const int dim = 4 * l32, m = dim / DSUB;
                        const int code = cv[(int64_t)tok * M + m];
                        v = *(const half4_t*)(cbv + (m * 256 + code) * DSUB + (dim % DSUB));
                    }
                }
                *(half4_t*)(s_rows + r * kD + 4 * l32) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // ---- P.V: tokens along k; transposed LDS reads turn row-major V rows into the B operand
            half8_t pa = *(const half8_t*)(s_p + (arow & 3) * 32 + 8 * kgrp);
            if (arow >= kNH) pa = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
            const uint32_t rows_off = (uint32_t)(L::a_rows + wave * 8192);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                half4_t vb[2];
#pragma unroll
                for (int hi = 0; hi < 2; ++hi) {
                    const int row = 8 * kgrp + 4 * hi + tj;
                    vb[hi] = lds_read_tr16(lsm, rows_off + (uint32_t)(row * kD + 16 * c + 4 * tq) * 2);
                }
                const half8_t bop = {vb[0][0], vb[0][1], vb[0][2], vb[0][3], vb[1][0], vb[1][1], vb[1][2], vb[1][3]};
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, bop, acc[c], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
        float l_sum[kNH];
#pragma unroll
        for (int h = 0; h < kNH; ++h) l_sum[h] = wave_sum(l_lane[h]);
        wg_merge_and_store<DSUB>(smem, m_ref, l_sum, acc, part_bg, aw, slots, nheads, L::a_red);
    }
}

// out[b][h] = sum_s acc_s 2^(m_s - m) / sum_s l_s 2^(m_s - m).  One 128-thread workgroup per (b, h).
__global__ __launch_bounds__(128) void decode_merge_kernel(const float* __restrict__ part, int slots,
                                                           half_t* __restrict__ out)
{
    const int bh = blockIdx.x, dim = threadIdx.x;
    const float* pb = part + (int64_t)bh * slots * (kD + 2);
    float m = kNegBig;
    for (int s = 0; s < slots; ++s) m = fmaxf(m, pb[s * (kD + 2) + kD]);
    float l = 0.f, a = 0.f;
    for (int s = 0; s < slots; ++s) {
        const float w = fast_exp2(pb[s * (kD + 2) + kD] - m);
        l += pb[s * (kD + 2) + kD + 1] * w;
        a += pb[s * (kD + 2) + dim] * w;
    }
    out[(int64_t)bh * kD + dim] = (half_t)(l > 0.f ? a / l : 0.f);
}

__global__ __launch_bounds__(128) void zero_out_kernel(half_t* out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (half_t)0.f;
}

// -------------------------------------------------------------------------------------------------
// Decode-time Anchor Score: p_hj = softmax_j(scale q_h . K_eff[j]) needs the final per-head
// log-sum-exp, so it is a two-pass scheme over the K codes with an fp32 lookup table (the fp16 table of
// the attention path is not accurate enough to rank tokens): pass 0 accumulates (max, sum) per split,
// pass 1 writes ans_v[j] = sum_h p_hj and ans_k[j] = sum_h p_hj (1 - p_hj) ||q_h||_2.
// -------------------------------------------------------------------------------------------------
struct DsParams {
    const half_t* q;
    const uint8_t* codes_k;
    const half_t* cb_k;
    const int32_t* idx_k;
    const half_t* rows_k;
    float* stat_part;      // [B][Hq][S][2]
    float* lse2;           // [B][Hq]
    float *ans_k, *ans_v;  // [B][Hkv][N]
    int64_t N, N_cap;
    int k_k;
    float c1;
    int Hq, Hkv, G, S;
    int64_t chunk;
};

template <int DSUB, int PASS>
__global__ __launch_bounds__(kDaThreads) void decode_ans_kernel(const DsParams p)
{
    constexpr int M = kD / DSUB;
    constexpr int CW = M / 4;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    float4_t* s_lut = (float4_t*)smem;                      // [M][256] x 4 heads fp32
    float* s_qf = (float*)(smem + M * 256 * 16);            // [4][128]
    float* s_red = s_qf + kNH * kD;                         // [waves][8]
    int* s_misc = (int*)(s_red + kDaWaves * 8);             // 16 ints
    uint32_t* s_mask = (uint32_t*)(s_misc + 16);            // bitmap of K-anchored tokens, 1024 words
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bg = blockIdx.x / p.S, sp = blockIdx.x % p.S;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int h0 = g * p.G;
    const half_t* qb = p.q + ((int64_t)b * p.Hq + h0) * kD;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;

    if (tid < kNH * kD) s_qf[tid] = ((tid >> 7) < p.G) ? (float)qb[tid] : 0.f;
    for (int i = tid; i < 1024; i += kDaThreads) s_mask[i] = 0u;
    if (wave < 2) {
        const int r = wave_lower_bound(idx_k, p.k_k, (int)(wave ? t1 : t0), lane);
        if (lane == 0) s_misc[wave] = r;
    }
    __syncthreads();
    {
        const half_t* cbk = p.cb_k + (size_t)g * 32768;
        for (int e = tid; e < M * 256; e += kDaThreads) {
            const int m = e >> 8;
            float4_t o;
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                float s = 0.f;
#pragma unroll
                for (int t = 0; t < DSUB; ++t) s = fmaf(s_qf[h * kD + m * DSUB + t], (float)cbk[e * DSUB + t], s);
                o[h] = s * p.c1;
            }
            s_lut[e] = o;
        }
    }
    for (int i = s_misc[0] + tid; i < s_misc[1]; i += kDaThreads) {
        const int rel = idx_k[i] - (int)t0;
        atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
    }
    float qn[kNH], lse[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) {
        float s = 0.f;
#pragma unroll 1
        for (int t = 0; t < kD; ++t) s = fmaf(s_qf[h * kD + t], s_qf[h * kD + t], s);
        qn[h] = sqrtf(s);
        lse[h] = (PASS == 1 && h < p.G) ? p.lse2[(int64_t)b * p.Hq + h0 + h] : 0.f;
    }
    __syncthreads();
    const int lo_k = s_misc[0], hi_k = s_misc[1];
    const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * M;
    float m_run[kNH], l_run[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) { m_run[h] = kNegBig; l_run[h] = 0.f; }

    for (int64_t tok = t0 + tid; tok < t1; tok += kDaThreads) {
        uint32_t kw[CW];
        if (CW == 2) { const uint2_t a = *(const uint2_t*)(ck + tok * M); kw[0] = a[0]; kw[1] = a[1]; }
        else {
#pragma unroll
            for (int i = 0; i < CW / 4; ++i) {
                const uint4_t a = *(const uint4_t*)(ck + tok * M + 16 * i);
#pragma unroll
                for (int e = 0; e < 4; ++e) kw[4 * i + e] = a[e];
            }
        }
        float s[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const uint32_t code = (kw[m >> 2] >> (8 * (m & 3))) & 255u;
            const float4_t e = s_lut[m * 256 + code];
#pragma unroll
            for (int h = 0; h < kNH; ++h) s[h] += e[h];
        }
        // K-anchored token: its score comes from the FP16 row (slot found in the slice of the list
        // that lies in this range)
        const int rel = (int)(tok - t0);
        if ((s_mask[rel >> 5] >> (rel & 31)) & 1u) {
            const int slot = find_sorted(idx_k + lo_k, hi_k - lo_k, (int)tok);
            const half_t* row = p.rows_k + ((int64_t)bg * p.k_k + lo_k + slot) * kD;
#pragma unroll
            for (int h = 0; h < kNH; ++h) s[h] = 0.f;
#pragma unroll 1
            for (int t = 0; t < kD; t += 8) {
                const half8_t v = *(const half8_t*)(row + t);
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int h = 0; h < kNH; ++h) s[h] = fmaf(s_qf[h * kD + t + e], (float)v[e], s[h]);
            }
#pragma unroll
            for (int h = 0; h < kNH; ++h) s[h] *= p.c1;
        }
        if (PASS == 0) {
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float m_new = fmaxf(m_run[h], s[h]);
                l_run[h] = l_run[h] * fast_exp2(m_run[h] - m_new) + fast_exp2(s[h] - m_new);
                m_run[h] = m_new;
            }
        } else {
            float av = 0.f, ak = 0.f;
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                if (h < p.G) {
                    const float a = fast_exp2(s[h] - lse[h]);
                    const float t = a * qn[h];
                    av += a;
                    ak += fmaf(-a, t, t);
                }
            }
            p.ans_v[(int64_t)bg * p.N + tok] = av;
            p.ans_k[(int64_t)bg * p.N + tok] = ak;
        }
    }
    if (PASS == 0) {
#pragma unroll
        for (int h = 0; h < kNH; ++h) {
            const float m_w = wave_max(m_run[h]);
            const float l_w = wave_sum(l_run[h] * fast_exp2(m_run[h] - m_w));
            if (lane == 0) { s_red[wave * 8 + h] = m_w; s_red[wave * 8 + 4 + h] = l_w; }
        }
        __syncthreads();
        if (tid < p.G) {
            float m = kNegBig;
            for (int w = 0; w < kDaWaves; ++w) m = fmaxf(m, s_red[w * 8 + tid]);
            float l = 0.f;
            for (int w = 0; w < kDaWaves; ++w) l += s_red[w * 8 + 4 + tid] * fast_exp2(s_red[w * 8 + tid] - m);
            float* dst = p.stat_part + (((int64_t)b * p.Hq + h0 + tid) * p.S + sp) * 2;
            dst[0] = m;
            dst[1] = l;
        }
    }
}

__global__ __launch_bounds__(64) void decode_ans_lse_kernel(const float* __restrict__ stat_part, int S,
                                                            float* __restrict__ lse2, int n_bh)
{
    const int bh = blockIdx.x * 64 + threadIdx.x;
    if (bh >= n_bh) return;
    float m = kNegBig;
    for (int s = 0; s < S; ++s) m = fmaxf(m, stat_part[((int64_t)bh * S + s) * 2]);
    float l = 0.f;
    for (int s = 0; s < S; ++s) l += stat_part[((int64_t)bh * S + s) * 2 + 1] * exp2f(stat_part[((int64_t)bh * S + s) * 2] - m);
    lse2[bh] = m + log2f(l);
}

// measurement aid: events to record around the next code-stream kernel launched from this host thread
thread_local hipEvent_t t_ev_start = nullptr, t_ev_stop = nullptr;

struct DaPlan {
    int S, A;
    int64_t chunk;
    size_t off_part, off_stat, off_lse, total;
};

DaPlan da_plan(const Geom& g, int64_t N, int64_t k_k, int64_t k_v, bool want_ans)
{
    DaPlan pl;
    const int64_t bg = (int64_t)g.B * g.Hkv;
    int64_t S = (256 + bg - 1) / bg;                 // about one stream workgroup per CU
    const int64_t max_S = (N + 1023) / 1024;         // at least ~1024 tokens per split
    if (S > max_S) S = max_S;
    if (S < 1) S = 1;
    int64_t chunk = (N + S - 1) / S;
    chunk = (chunk + 63) / 64 * 64;
    if (chunk > 32768) chunk = 32768;
    if (chunk < 64) chunk = 64;
    pl.chunk = chunk;
    pl.S = (int)((N + chunk - 1) / chunk);
    if (pl.S < 1) pl.S = 1;
    const int64_t tiles = (k_k + k_v + 31) / 32;
    pl.A = (int)((tiles + kAnchorTilesPerWg - 1) / kAnchorTilesPerWg);
    size_t off = 0;
    pl.off_part = off; off += align_up((size_t)g.B * g.Hq * (pl.S + pl.A) * (kD + 2) * sizeof(float));
    pl.off_stat = off; off += want_ans ? align_up((size_t)g.B * g.Hq * pl.S * 2 * sizeof(float)) : 0;
    pl.off_lse = off;  off += align_up((size_t)g.B * g.Hq * sizeof(float));
    pl.total = off;
    return pl;
}

}  // namespace

int decode_num_splits(const Geom& g, int64_t N) { return da_plan(g, N, 0, 0, false).S; }

void decode_profile_next(hipEvent_t start, hipEvent_t stop)
{
    t_ev_start = start;
    t_ev_stop = stop;
}

size_t decode_workspace_bytes(const Geom& g, int64_t N, int64_t k_k, int64_t k_v, bool want_ans)
{
    return da_plan(g, N, k_k, k_v, want_ans).total;
}

template <int DSUB>
static hipError_t launch_decode_t(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st)
{
    const bool want_ans = a.ans_k || a.ans_v;
    const DaPlan pl = da_plan(g, a.N, a.k_k, a.k_v, want_ans);
    char* w = (char*)ws;
    float* part = (float*)(w + pl.off_part);
    float* lse2 = (float*)(w + pl.off_lse);
    DaParams p;
    p.q = a.q; p.codes_k = a.codes_k; p.codes_v = a.codes_v; p.cb_k = a.cb_k; p.cb_v = a.cb_v;
    p.idx_k = a.idx_k; p.idx_v = a.idx_v; p.rows_k = a.rows_k; p.rows_v = a.rows_v;
    p.part = part; p.N = a.N; p.N_cap = a.N_cap; p.k_k = (int)a.k_k; p.k_v = (int)a.k_v;
    p.c1 = a.scale * kLog2e; p.Hq = g.Hq; p.Hkv = g.Hkv; p.G = g.G; p.S = pl.S; p.A = pl.A; p.chunk = pl.chunk;
    const size_t shmem = Lds<DSUB>::total;
    hipError_t e = hipFuncSetAttribute((const void*)decode_attn_kernel<DSUB>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((int64_t)g.B * g.Hkv * (pl.S + pl.A));
    if (t_ev_start) (void)hipEventRecord(t_ev_start, st);
    hipLaunchKernelGGL(decode_attn_kernel<DSUB>, dim3(grid), dim3(kDaThreads), shmem, st, p);
    if (t_ev_stop) (void)hipEventRecord(t_ev_stop, st);
    t_ev_start = t_ev_stop = nullptr;
    hipLaunchKernelGGL(decode_merge_kernel, dim3((unsigned)(g.B * g.Hq)), dim3(128), 0, st, part, pl.S + pl.A, a.out);
    if (want_ans) {
        DsParams d;
        d.q = a.q; d.codes_k = a.codes_k; d.cb_k = a.cb_k; d.idx_k = a.idx_k; d.rows_k = a.rows_k;
        d.stat_part = (float*)(w + pl.off_stat); d.lse2 = lse2; d.ans_k = a.ans_k; d.ans_v = a.ans_v;
        d.N = a.N; d.N_cap = a.N_cap; d.k_k = (int)a.k_k; d.c1 = p.c1; d.Hq = g.Hq; d.Hkv = g.Hkv; d.G = g.G;
        d.S = pl.S; d.chunk = pl.chunk;
        const size_t sh2 = (size_t)g.M * 256 * 16 + kNH * kD * 4 + kDaWaves * 32 + 64 + 4096;
        e = hipFuncSetAttribute((const void*)decode_ans_kernel<DSUB, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh2);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)decode_ans_kernel<DSUB, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh2);
        if (e != hipSuccess) return e;
        const unsigned grid2 = (unsigned)((int64_t)g.B * g.Hkv * pl.S);
        hipLaunchKernelGGL((decode_ans_kernel<DSUB, 0>), dim3(grid2), dim3(kDaThreads), sh2, st, d);
        hipLaunchKernelGGL(decode_ans_lse_kernel, dim3((unsigned)((g.B * g.Hq + 63) / 64)), dim3(64), 0, st,
                           d.stat_part, pl.S, lse2, g.B * g.Hq);
        hipLaunchKernelGGL((decode_ans_kernel<DSUB, 1>), dim3(grid2), dim3(kDaThreads), sh2, st, d);
    }
    return hipGetLastError();
}

hipError_t launch_decode_attn(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st)
{
    if (a.N == 0) {
        const int64_t n = (int64_t)g.B * g.Hq * kD;
        if (n == 0) return hipSuccess;
        hipLaunchKernelGGL(zero_out_kernel, dim3((unsigned)((n + 127) / 128)), dim3(128), 0, st, a.out, n);
        return hipGetLastError();
    }
    if (g.d == 4) return launch_decode_t<4>(g, a, ws, st);
    if (g.d == 8) return launch_decode_t<8>(g, a, ws, st);
    return launch_decode_t<16>(g, a, ws, st);
}

}  // namespace antkv
