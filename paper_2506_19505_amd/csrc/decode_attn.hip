// Decode attention over VQ codes + FP16 anchor tokens (paper Sec. 2.1 Attn with one query row; Sec. 3,
// Fig. 2(b): anchor tokens stay FP16, every other token is read from its codes), and the decode-time
// Anchor Score (Sec. 3.2 last paragraph: Eq. (4) evaluated for the single decode query).
//
// A workgroup (16 waves) owns a contiguous token range of one (sequence, KV head).
//
//  prologue  build the q.centroid lookup table LUT[code][slot][head] (15-bit fixed point stored as two signed
//            bytes, pre-multiplied by scale*log2e), copy the V codebook into LDS code-major, mark the anchored
//            tokens of the range in an LDS bitmap.  The table has 32 eight-byte slots per code row (= all 64
//            LDS banks); slot j holds sub-space j mod M.  Lane l reads slot (step XOR (l mod 32)) at every
//            step, i.e. it walks the sub-spaces in its own XOR-permuted order: the 32 lanes that the LDS
//            serves per clock always hit 32 different bank pairs, whatever the codes are (random gathers
//            would run at a third of that).
//  anchors   the (sequence, KV head)'s anchor lists are cut into 32-entry tiles dealt round-robin to the
//            workgroups (balanced by list index, not by position: anchors cluster at the head and tail of a
//            context); inside a workgroup whichever wave is free takes the next tile before it joins the
//            stream.  K_eff chunks (the FP16 row, or the de-quantised codes when only V of that token is
//            anchored) go straight from global memory into the MFMA operand; V_eff rows pass through the
//            wave's staging area for the transposed reads.
//  stream    waves pull 64-token tiles from a shared counter, code loads running one tile ahead:
//      K side  one lane per token: 16-byte coalesced code loads, one 8-byte LUT gather per sub-space
//              serves the group's four query heads.  The gathered entries are the row operand of an int8 MFMA
//              whose column operand is a constant block-diagonal matrix: it sums the entries exactly and, at
//              the same time, transposes the result: lane (4 c + h, k-group g) ends up with head h's scores of
//              the four tokens 16 c + 4 g + 0..3, which is exactly where the sparse operand of P.V wants them;
//      softmax base-2 online softmax against a lazily updated reference maximum (the wave only pays
//              the cross-lane reduction when some score exceeds the reference); the four fp16 weights of a
//              lane, zero-extended, are the P.V operand as they stand: no trip through LDS;
//      V side  P.V runs on the 2:4-sparse MFMA, all 16 rows in use (rows = slab class x head, see the comment at
//              sm_idx).  The four positions of a group of the k axis are four different tokens, each with the
//              16-channel slab (class + rotation) mod 4 of one half of the row, and eight MFMAs per tile (four
//              rotations x two halves, an accumulator each) take every token through all eight slabs.  The V
//              code bytes reach the lanes that need them through the wave's staging area, rotated by the
//              token's class so that the reader's byte position is a constant; V centroids are fetched with
//              ds_read_b64_tr_b16, whose lane transposition yields the dense MFMA operand.
//      Tokens that have an FP16 anchor row (for K or for V) are masked out of the stream.
//
// The workgroup merges its waves and writes one partial (reference max, sum, accumulator) per query head;
// the last workgroup of a (sequence, KV head) to finish merges the partials by log-sum-exp and rounds once
// to fp16: the whole step is one kernel.
#include "common.h"

#include <atomic>

namespace antkv {

namespace {

constexpr int kDaWaves = 16;
constexpr int kDaThreads = kDaWaves * 64;
constexpr int kNH = 4;                 // query-head slots per workgroup (group size G <= 4)
constexpr float kPShift = 8.0f;        // P is scaled by 2^8 so that small weights stay normal in fp16
constexpr float kLutMax = 16256.0f;    // largest table magnitude: 127 * 128, so that both bytes of an entry fit int8
constexpr int kPStride = 72;           // fp16 elements between the heads of a wave's P tile (64 + pad against bank conflicts)
// per-wave staging.  Anchor tiles: fp16 P tile, then 1 KB of V rows.  Stream: the V code bytes of a tile (up to 1 KB).
constexpr int kStgBytes = 1664;
static_assert(4 * kPStride * 2 + 1024 <= kStgBytes && kStgBytes % 16 == 0, "anchor staging fits the per-wave area");
constexpr float kEmptyRef = -1.0e4f;   // softmax reference before any token was seen: finite, below every real score,
                                       // and far above the masked score kNegBig so that exp2(masked - ref) is 0

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) short4_t lds_short4;
typedef __attribute__((address_space(3))) uint2_t lds_uint2;

__device__ __forceinline__ half4_t lds_read_tr16(const lds_char* base, uint32_t off)
{
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(base + off));
    return __builtin_bit_cast(half4_t, v);
}
// same, from an absolute LDS byte address (lets the caller fold the array base into a per-lane constant
// and keeps compile-time addends in the instruction's immediate offset)
__device__ __forceinline__ half4_t lds_read_tr16_abs(uint32_t addr)
{
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(uintptr_t)addr);
    return __builtin_bit_cast(half4_t, v);
}

template <int SRC>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, SRC * 0x55, 0xf, 0xf, true);
}

__device__ __forceinline__ uint32_t quad_bcast_sel(uint32_t x, int src)
{
    switch (src) {
    case 0: return quad_bcast<0>(x);
    case 1: return quad_bcast<1>(x);
    case 2: return quad_bcast<2>(x);
    default: return quad_bcast<3>(x);
    }
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

// max / sum over each row of 16 lanes, result in all 16 lanes of the row
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true)));
    return v;
}
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true));
    return v;
}
__device__ __forceinline__ float lane_bcast(float v, int src_lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src_lane));
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

// two searches in lockstep (key_a <= key_b): the probe loads of a round are issued together, so the pair costs
// the latency of one search
__device__ void wave_lower_bound2(const int32_t* __restrict__ arr, int n, int key_a, int key_b, int lane,
                                  int& res_a, int& res_b)
{
    int lo_a = 0, hi_a = n, lo_b = 0, hi_b = n;
    while (hi_a > lo_a || hi_b > lo_b) {
        const int st_a = (hi_a - lo_a + 63) >> 6, st_b = (hi_b - lo_b + 63) >> 6;
        const int p_a = lo_a + lane * st_a, p_b = lo_b + lane * st_b;
        const int v_a = (p_a < hi_a) ? arr[p_a] : 0x7fffffff;
        const int v_b = (p_b < hi_b) ? arr[p_b] : 0x7fffffff;
        if (hi_a > lo_a) {
            const int c = __builtin_popcountll(__ballot(v_a < key_a));
            if (c == 0) hi_a = lo_a;
            else {
                const int nlo = lo_a + (c - 1) * st_a + 1, nhi = lo_a + c * st_a;
                lo_a = nlo;
                hi_a = nhi < hi_a ? nhi : hi_a;
                if (st_a == 1) hi_a = lo_a;
            }
        }
        if (hi_b > lo_b) {
            const int c = __builtin_popcountll(__ballot(v_b < key_b));
            if (c == 0) hi_b = lo_b;
            else {
                const int nlo = lo_b + (c - 1) * st_b + 1, nhi = lo_b + c * st_b;
                lo_b = nlo;
                hi_b = nhi < hi_b ? nhi : hi_b;
                if (st_b == 1) hi_b = lo_b;
            }
        }
    }
    res_a = lo_a;
    res_b = lo_b;
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
    float* part;                // [B][Hq][S][kD + 2]
    half_t* out;                // [B][Hq][kD]
    unsigned long long* done;   // [B][Hkv] arrival words (launch tag << 32 | count); the last workgroup of a (b, g) merges
    unsigned int tag;           // this launch's tag: words carrying another tag count as zero, so no clearing pass
    int64_t N, N_cap;
    int k_k, k_v;
    float c1;                   // scale * log2(e)
    int Hq, Hkv, G;
    int S;                      // workgroups (token ranges) per (b, g)
    int64_t chunk;              // tokens per range (multiple of 64)
};

// LDS layout (bytes); the final merge re-uses the table area.  The two tables sit at multiples of 64 KB so
// that a gather address is (table base | code << 8 | byte inside the code's 256-byte row).
template <int DSUB>
struct Lds {
    static constexpr int M = kD / DSUB;
    static constexpr int lut = 0;                                  // [256 codes][32 slots][4 x (lo, hi) bytes] = 64 KB
    static constexpr int cbv = lut + 65536;                        // [256 codes][M][DSUB] fp16 = 64 KB (a 256-byte row per code)
    static constexpr int pst = cbv + 65536;                        // [waves] staging (P tile + V code words / anchor V rows)
    static constexpr int mrg = 0;                                  // merge: [waves][4 classes][128 channels][4 heads] fp32 = 128 KB (the two tables are free by then)
    static constexpr int qh = pst + kDaWaves * kStgBytes;          // [4][128] fp16 (MFMA operand source)
    static constexpr int red = qh + 1024;                          // [waves][8] fp32 + 16 ints
    static constexpr int mask = red + kDaWaves * 32 + 64;          // bitmap over the token range
    static constexpr int mask_words = 1024;                        // up to 32768 tokens per range
    static constexpr int total = mask + mask_words * 4;
    static_assert(total <= 163840, "LDS budget of one CU");
};

// Merge the waves' (m_ref, l, acc) into one partial and write it.  acc[a][rho] is in the C layout of the class-structured
// sparse MFMA: register h of a lane (cls = lane / 16, n = lane % 16) is head h, channel 16 (4 a + (cls + rho) % 4) + n,
// summed over the tokens of class cls only, so the four classes (and the waves) still have to be added up.
template <int DSUB>
__device__ void wg_merge_and_store(char* smem, float (&m_ref)[kNH], float (&l_sum)[kNH], float4_t (&acc)[2][4],
                                   float* __restrict__ part_bg, int slot, int slots, int nheads)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float* s_red = (float*)(smem + Lds<DSUB>::red);
    __syncthreads();   // everyone is done with the tables and the staging area
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < kNH; ++h) { s_red[wave * 8 + h] = m_ref[h]; s_red[wave * 8 + 4 + h] = l_sum[h]; }
    }
    __syncthreads();
    static_assert(kDaWaves <= 16, "one row of 16 lanes covers the waves");
    float m_all[kNH], l_all[kNH];
    {
        const int hh = lane >> 4, ws = lane & 15;               // this lane looks at (head hh, wave ws)
        const float m_w = (ws < kDaWaves) ? s_red[ws * 8 + hh] : kNegBig;
        const float l_w = (ws < kDaWaves) ? s_red[ws * 8 + 4 + hh] : 0.f;
        const float m_r = row16_max(m_w);
        const float l_r = row16_sum(l_w * fast_exp2(m_w - m_r));
#pragma unroll
        for (int h = 0; h < kNH; ++h) { m_all[h] = lane_bcast(m_r, 16 * h); l_all[h] = lane_bcast(l_r, 16 * h); }
    }
    float4_t f;
#pragma unroll
    for (int h = 0; h < kNH; ++h) f[h] = fast_exp2(m_ref[h] - m_all[h]);
    static_assert(kDaWaves * 4 * kD * 16 <= 131072, "the merge area is the two tables");
    float4_t* s_mrg = (float4_t*)(smem + Lds<DSUB>::mrg);            // [wave][class][channel] x 4 heads
    const int cls = lane >> 4, n = lane & 15;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int rho = 0; rho < 4; ++rho)
            s_mrg[(wave * 4 + cls) * kD + 16 * (4 * a + ((cls + rho) & 3)) + n] = acc[a][rho] * f;
    __syncthreads();
    if (tid < kNH * kD) {
        const int h = tid & 3, dim = tid >> 2;                   // consecutive threads read consecutive dwords
        const float* src = (const float*)s_mrg + dim * 4 + h;
        float s4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
        for (int w = 0; w < kDaWaves * 4; w += 4) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s4[u] += src[(w + u) * kD * 4];
        }
        if (h < nheads) {
            const float s = (s4[0] + s4[1]) + (s4[2] + s4[3]);
            float* dst = part_bg + ((int64_t)h * slots + slot) * (kD + 2);
            // Device-scope stores: they write through this die's L2, so the merging workgroup (possibly
            // on another die) can read them without any cache write-back.
            __hip_atomic_store(dst + dim, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (dim == 0) {
                __hip_atomic_store(dst + kD, m_all[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(dst + kD + 1, l_all[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

template <int DSUB>
__global__ __launch_bounds__(kDaThreads) void decode_attn_kernel(const DaParams p)
{
    constexpr int M = kD / DSUB;
    constexpr int CW = M / 4;                          // code dwords per token
    static_assert(kDaWaves == 16, "the table build gives each of 16 waves 16 of the 256 codes");
    using L = Lds<DSUB>;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    const lds_char* lsm = (const lds_char*)smem_u4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups go to the 8 XCDs round-robin by their id; remap so that the S workgroups of one (sequence, KV head)
    // sit on one XCD and share its L2 for the codebooks and the anchor lists.
    const int wg = (gridDim.x & 7) == 0 ? (int)((blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3)) : (int)blockIdx.x;
    const int bg = wg / p.S, sp = wg % p.S;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int nheads = p.G;               // <= kNH
    const int h0 = g * p.G;
    float* part_bg = p.part + ((int64_t)b * p.Hq + h0) * p.S * (kD + 2);
    const half_t* qb = p.q + ((int64_t)b * p.Hq + h0) * kD;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const int32_t* idx_v = p.idx_v + (int64_t)bg * p.k_v;
    const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * M;
    const uint8_t* cv = p.codes_v + (int64_t)bg * p.N_cap * M;
    const half_t* cbk = p.cb_k + (size_t)g * 32768;
    const half_t* cbv = p.cb_v + (size_t)g * 32768;
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;
    // Arrival word of this (b, g): (launch tag << 32 | arrivals).  A word left by an earlier launch (another tag,
    // or this tag with all S arrivals when a captured launch is replayed) is replaced by (tag, 0) now, by
    // whichever workgroup gets there first, so that the arrival at the end is a single fetch-add.  Launches
    // that share a workspace do not overlap, hence nobody of an earlier launch still touches the word.
    // (the word is loaded here, with the other loads of the prologue, and swapped once those have landed)
    unsigned long long done_seen = 0ull;
    if (tid == 0) done_seen = __hip_atomic_load(&p.done[bg], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // MFMA lane coordinates
    const int kgrp = lane >> 4;           // tr block / k group
    const int tj = (lane >> 2) & 3;       // token within a group of four
    const int tq = lane & 3;              // 8-byte chunk of a 32-byte channel slab / quad lane
    const int arow = lane & 15;           // A-operand row (head) / C column (channel)

    int* s_misc = (int*)(smem + L::red + kDaWaves * 32);
    uint32_t* s_mask = (uint32_t*)(smem + L::mask);

    // ================================================================================== prologue
    {
        // all global loads of the prologue are issued before anything waits on them.
        // the small loads go first: the first barrier then waits for them only, and the two 64 KB tables
        // keep streaming in behind it
        half_t qv16 = (half_t)0.f;
        if (tid < kNH * kD && (tid >> 7) < nheads) qv16 = qb[tid];
        // anchored positions of this range: short lists are scanned whole (one load latency), long lists are
        // cut to the range by a cooperative search first (a few dependent load latencies)
        constexpr int kScanRounds = 4;
        constexpr int kScanMax = kScanRounds * kDaThreads;
        const bool scan_k = p.k_k <= kScanMax, scan_v = p.k_v <= kScanMax;
        int scan_val[2][kScanRounds];
#pragma unroll
        for (int i = 0; i < kScanRounds; ++i) {
            const int j = tid + i * kDaThreads;
            scan_val[0][i] = -1;
            scan_val[1][i] = -1;
            if (scan_k && i * kDaThreads < p.k_k) scan_val[0][i] = (j < p.k_k) ? idx_k[j] : -1;   // uniform skip of empty rounds
            if (scan_v && i * kDaThreads < p.k_v) scan_val[1][i] = (j < p.k_v) ? idx_v[j] : -1;
        }
        if (wave < 4) {
            const int32_t* arr = (wave < 2) ? idx_k : idx_v;
            const int n = (wave < 2) ? p.k_k : p.k_v;
            int r = 0;
            if (!((wave < 2) ? scan_k : scan_v)) r = wave_lower_bound(arr, n, (int)((wave & 1) ? t1 : t0), lane);
            if (lane == 0) s_misc[wave] = r;
        }
        // The q.centroid table is one small matrix product per sub-space, batched on the MFMA by making the
        // query operand block-diagonal: an MFMA takes 16 codes (columns) and four sub-spaces; k-group kg of the
        // centroid operand holds sub-space kg's centroid (or half / two of them for d = 16 / 4), and row 4 m' + h of
        // the query operand is q_h's matching slice in k-group m' and zero elsewhere.  C then holds, in lane
        // (code, block m'), the four heads' products for (sub-space of block m', code): one table entry per lane.
        constexpr int NJ = (DSUB == 4) ? 8 : 4;            // MFMAs per wave; each wave owns 16 codes
        const int l_code = 16 * wave + (lane & 15);        // this lane's code (column)
        const int l_mp = (lane & 15) >> 2, l_h = lane & 3; // query-operand row = 4 m' + h
        uint4_t opb[4], opa[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            opa[j] = uint4_t{0u, 0u, 0u, 0u};
            if constexpr (DSUB == 8) {
                opb[j] = *(const uint4_t*)(cbk + ((4 * j + kgrp) * 256 + l_code) * 8);
                if (kgrp == l_mp && l_h < nheads) opa[j] = *(const uint4_t*)(qb + l_h * kD + (4 * j + l_mp) * 8);
            } else if constexpr (DSUB == 16) {
                opb[j] = *(const uint4_t*)(cbk + ((2 * j + (kgrp >> 1)) * 256 + l_code) * 16 + 8 * (kgrp & 1));
                if ((kgrp >> 1) == l_mp && l_h < nheads)
                    opa[j] = *(const uint4_t*)(qb + l_h * kD + (2 * j + l_mp) * 16 + 8 * (kgrp & 1));
            } else {
                const uint2_t lo = *(const uint2_t*)(cbk + ((8 * j + 2 * kgrp) * 256 + l_code) * 4);
                const uint2_t hi = *(const uint2_t*)(cbk + ((8 * j + 2 * kgrp + 1) * 256 + l_code) * 4);
                opb[j] = uint4_t{lo[0], lo[1], hi[0], hi[1]};
                if (kgrp == l_mp && l_h < nheads) opa[j] = *(const uint4_t*)(qb + l_h * kD + (8 * j + 2 * l_mp) * 4);
            }
        }
        // V codebook: LDS holds it code-major ([code][m][DSUB], a 256-byte row per code), so 16-byte chunk ci of
        // the LDS image comes from a permuted place of the sub-space-major global array
        uint4_t vcopy[4096 / kDaThreads];
#pragma unroll
        for (int i = 0; i < 4096 / kDaThreads; ++i) {
            const int ci = tid + i * kDaThreads, code = ci >> 4, w16 = ci & 15;
            if constexpr (DSUB == 8) {
                vcopy[i] = ((const uint4_t*)cbv)[w16 * 256 + code];
            } else if constexpr (DSUB == 16) {
                vcopy[i] = ((const uint4_t*)cbv)[((w16 >> 1) * 256 + code) * 2 + (w16 & 1)];
            } else {
                const uint2_t lo = ((const uint2_t*)cbv)[(2 * w16) * 256 + code], hi = ((const uint2_t*)cbv)[(2 * w16 + 1) * 256 + code];
                vcopy[i] = uint4_t{lo[0], lo[1], hi[0], hi[1]};
            }
        }
        if (tid < kNH * kD) ((half_t*)(smem + L::qh))[tid] = qv16;
        for (int i = tid; i < L::mask_words; i += kDaThreads) s_mask[i] = 0u;
        if (tid == 0) { s_misc[8] = 0; s_misc[9] = 0; }          // next stream tile, next anchor tile of this workgroup
        __syncthreads();
        if (tid == 0 && ((unsigned int)(done_seen >> 32) != p.tag || (unsigned int)done_seen >= (unsigned int)p.S))
            __hip_atomic_compare_exchange_strong(&p.done[bg], &done_seen, (unsigned long long)p.tag << 32, __ATOMIC_RELAXED,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // bitmap of anchored tokens in this range
        const uint32_t range_len = (uint32_t)(t1 - t0);
#pragma unroll
        for (int w2 = 0; w2 < 2; ++w2)
#pragma unroll
            for (int i = 0; i < kScanRounds; ++i) {
                if (i * kDaThreads < (w2 ? p.k_v : p.k_k)) {
                    // unsigned compare: positions below t0 (and the -1 filler) wrap to huge values
                    const uint32_t rel = (uint32_t)scan_val[w2][i] - (uint32_t)t0;
                    if (scan_val[w2][i] >= 0 && rel < range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
                }
            }
        // positions between the end of the range and the end of its last tile count as anchored: the stream skips them
        if (tid < 64) {
            const uint32_t rel = ((range_len - 1u) & ~63u) + (uint32_t)tid;
            if (rel >= range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
        }
        if (!scan_k) {
            for (int i = s_misc[0] + tid; i < s_misc[1]; i += kDaThreads) {
                const int rel = idx_k[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        if (!scan_v) {
            for (int i = s_misc[2] + tid; i < s_misc[3]; i += kDaThreads) {
                const int rel = idx_v[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        // LUT[m][c][h] = c1 * q_h[m*d : (m+1)*d] . cb_k[g][m][c], stored as fixed point with one scale per head
        // (quantum = max|LUT_h| / 16256): the per-token sum over sub-spaces is then exact integer arithmetic and
        // the table error is uniform instead of growing with the entry's magnitude as it would in fp16.
        // An entry is two signed bytes (lo, -hi) with value lo + 128 * hi, so that the int8 MFMA of the stream
        // loop can sum entries with the weights (1, -128).
        float val[NJ][kNH];
        float amax[kNH] = {0.f, 0.f, 0.f, 0.f};
        const bool ent_on = (DSUB != 16) || kgrp < 2;       // d = 16: only blocks 0 and 1 carry sub-spaces
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint4_t a4 = opa[(DSUB == 4) ? (j >> 1) : j];
            if constexpr (DSUB == 4) {                       // sub-space 2 m' + u of the pair lives in half u of the slice
                if (j & 1) { a4[0] = 0u; a4[1] = 0u; } else { a4[2] = 0u; a4[3] = 0u; }
            }
            const float4_t c4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                __builtin_bit_cast(half8_t, a4), __builtin_bit_cast(half8_t, opb[(DSUB == 4) ? (j >> 1) : j]),
                float4_t{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                val[j][h] = c4[h] * p.c1;
                if (ent_on) amax[h] = fmaxf(amax[h], fabsf(val[j][h]));
            }
        }
        float* s_red = (float*)(smem + L::red);
#pragma unroll
        for (int h = 0; h < kNH; ++h) {
            const float wm = wave_max_uniform(amax[h]);
            if (lane == 0) s_red[wave * 8 + h] = wm;
        }
        __syncthreads();
        float inv_q[kNH];
        {
            const int hh = lane >> 4, ws = lane & 15;
            const float r_r = row16_max((ws < kDaWaves) ? s_red[ws * 8 + hh] : 0.f);
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float r = lane_bcast(r_r, 16 * h);
                // the table quantum is parked in LDS until the stream starts (keeps registers free for the anchors)
                if (tid == 0) ((float*)s_misc)[12 + h] = (r > 0.f) ? r / kLutMax : 1.0f;
                inv_q[h] = (r > 0.f) ? kLutMax / r : 0.f;
            }
        }
        uint2_t* s_lut = (uint2_t*)(smem + L::lut);
        uint2_t ent[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint32_t hw[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const int qv = (int)rintf(val[j][h] * inv_q[h]);     // |qv| <= kLutMax
                const int hi = (qv + 64) >> 7;                          // qv = lo + 128 * hi, lo in [-64, 63]
                const int lo = qv - 128 * hi;
                hw[h] = ((uint32_t)lo & 0xffu) | (((uint32_t)(-hi) & 0xffu) << 8);
            }
            ent[j] = uint2_t{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16)};
        }
        // The lanes of a block hold the same sub-space for 16 different codes, i.e. 16 rows at the same bank.  In
        // round r a lane therefore stores entry (r + code) mod NJ, and starts with copy (code / 4) mod REPS of it:
        // the 32 lanes of an LDS pass then spread over 16 or 32 different slots.
        constexpr int REPS = 32 / M;
        if (ent_on) {
#pragma unroll
            for (int r = 0; r < NJ; ++r) {
                const int j = (r + lane) & (NJ - 1);
                uint2_t e = ent[0];
#pragma unroll
                for (int jj = 1; jj < NJ; ++jj) e = (j == jj) ? ent[jj] : e;
                const int m = (DSUB == 8) ? 4 * j + kgrp : (DSUB == 16 ? 2 * j + kgrp : 8 * (j >> 1) + 2 * kgrp + (j & 1));
#pragma unroll
                for (int rep = 0; rep < REPS; ++rep)
                    s_lut[l_code * 32 + m + M * ((rep + (lane >> 2)) & (REPS - 1))] = e;
            }
        }
        // the V table is not needed before the first P.V: its loads had the whole table build to land
        {
            uint4_t* dst = (uint4_t*)(smem + L::cbv);
#pragma unroll
            for (int i = 0; i < 4096 / kDaThreads; ++i) dst[tid + i * kDaThreads] = vcopy[i];
        }
    }
    __syncthreads();

    // m_ref: reference maximum per head (the same in every lane).  acc[a][rho]: see sm_idx below.
    float m_ref[kNH];
    float4_t acc[2][4];
#pragma unroll
    for (int h = 0; h < kNH; ++h) m_ref[h] = kEmptyRef;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int rho = 0; rho < 4; ++rho) acc[a][rho] = float4_t{0.f, 0.f, 0.f, 0.f};
    float l_own = 0.f;                                            // sum of weights, head lane % 4, this lane's share
    half_t* s_p = (half_t*)(smem + L::pst + wave * kStgBytes);    // this wave's P tile, [4][kPStride] fp16
    uint32_t* s_cw = (uint32_t*)(s_p + 4 * kPStride);             // this wave's V code words, 512 bytes

    // P.V runs on the 2:4-sparse MFMA (16x16x64 f16).  Its 64 k positions form 16 groups of four; the position
    // inside a group is the class, and row 4 cls + h of the sparse operand keeps, in every group, only the
    // position of its own class: a softmax weight of head h.  All 16 rows carry useful work, and the compressed
    // operand is just four zero-extended fp16 weights per lane (the index register, a per-lane constant, says
    // where they sit).  What a position means differs between the two users:
    //   anchor tiles  the four positions of a group are the four 16-channel slabs 4 a + cls of ONE item; output row
    //                 (cls, h) of MFMA a accumulates slab 4 a + cls;
    //   stream        the four positions of a group are FOUR tokens (one per class), position cls carrying slab
    //                 4 a + (cls + rho) % 4 of its token; MFMA (a, rho) accumulates into acc[a][rho], whose row
    //                 (cls, h) is therefore slab 4 a + (cls + rho) % 4 summed over the tokens of class cls.
    // With rho = 0 the two meanings of a row agree, so anchor tiles add into acc[a][0].
    // Operand geometry: compressed dword p of a lane in k-group ga pairs with the dense operand's k-group
    // 2 (ga % 2) + p / 2, elements 4 (2 (ga / 2) + p % 2) .. + 3.
    const int sm_idx = (int)(0x1111u * (uint32_t)(tj | ((tj ^ 1) << 2)));
    // P-tile slot of the (token, head) weights so that the four weights a lane needs are contiguous:
    // the item in dense k-group gb, element quad e4 of sparse MFMA i -> slot 16 i + 4 ga + p
    auto p_slot = [](int i, int gb_, int e4) {
        return 16 * i + 4 * ((gb_ >> 1) + 2 * (e4 >> 1)) + 2 * (gb_ & 1) + (e4 & 1);
    };
    auto load_pa = [&](int i) -> half8_t {
        const uint2_t w2 = *(const uint2_t*)(s_p + (lane & 3) * kPStride + 16 * i + 4 * kgrp);
        const uint4_t a4 = {w2[0] & 0xffffu, w2[0] >> 16, w2[1] & 0xffffu, w2[1] >> 16};
        return __builtin_bit_cast(half8_t, a4);
    };

    // ================================================================================== anchors
    const int n_items = p.k_k + p.k_v;                    // K-anchor entries, then V-anchor entries
    const int n_atiles = (n_items + 31) >> 5;
    // An anchor tile is a chain of dependent loads (lists, cross membership, rows) that leaves the CU idle if every
    // wave of the workgroup sits in one at the same time.  So only some waves take anchor tiles, up to five each,
    // while the others start streaming at once: 2, 4, 8 or all 16 waves, by the number of tiles of the workgroup.
    int anchor_waves = 2;
    {
        const int tiles_wg = (n_atiles + p.S - 1) / p.S;
        while (anchor_waves < kDaWaves && 5 * anchor_waves < tiles_wg) anchor_waves <<= 1;
    }
    if (n_atiles > 0 && (wave & (kDaWaves / anchor_waves - 1)) == 0) {
        float l_lane[kNH] = {0.f, 0.f, 0.f, 0.f};                        // per-lane shares of the weight sums, per head
        const half_t* s_qh = (const half_t*)(smem + L::qh);               // Q as MFMA A operand: row = head
        half_t* s_vrows = (half_t*)s_cw;                                  // [8 items][64 channels] fp16
        int* s_win = (int*)s_cw;                                          // 64 ints in the code-word area
        const uint32_t rows_off = (uint32_t)(L::pst + wave * kStgBytes + 4 * kPStride * 2);
        for (;;) {
            // tiles of the (b, g) lists are dealt round-robin to the workgroups; this workgroup's tiles are
            // handed out to its anchor waves through a counter
            int lt = 0;
            if (lane == 0) lt = atomicAdd(&s_misc[9], 1);
            lt = __builtin_amdgcn_readfirstlane(lt);
            const int t = sp + p.S * lt;
            if (t >= n_atiles) break;
            const int item0 = t * 32;
            // lanes 0..31 each own one item of the tile
            const bool is_k_tile_lane = (item0 + lane) < p.k_k;
            int my_tok = 0x7fffffff, my_kslot = -1, my_vslot = -1, my_valid = 0;
            if (lane < 32) {
                const int it = item0 + lane;
                if (it < p.k_k) { my_tok = idx_k[it]; my_kslot = it; my_valid = 1; }
                else if (it < n_items) { my_tok = idx_v[it - p.k_k]; my_vslot = it - p.k_k; my_valid = 1; }
            }
            // Cross membership: a K item looks its token up in idx_v (is its V row FP16 too?), a V item in idx_k
            // (if found there, the token is handled as a K item and this entry is skipped).  A tile can straddle
            // the two lists, so both lookups are run; each is a cooperative search for the window of the other
            // list that can contain the tile's tokens, then a search inside the window from LDS.
#pragma unroll 1
            for (int side = 0; side < 2; ++side) {
                const int32_t* arr = side ? idx_k : idx_v;
                const int n = side ? p.k_k : p.k_v;
                const bool mine = my_valid && (side ? !is_k_tile_lane : is_k_tile_lane) && lane < 32;
                const unsigned long long act = __ballot(mine);
                if (act == 0ull || n == 0) continue;
                const int l_first = __builtin_ctzll(act), l_last = 63 - __builtin_clzll(act);
                const int tok_first = __shfl(my_tok, l_first, 64), tok_last = __shfl(my_tok, l_last, 64);
                int w_lo, w_hi;
                wave_lower_bound2(arr, n, tok_first, tok_last + 1, lane, w_lo, w_hi);
                int found = -1;
                if (w_hi - w_lo <= 64) {
                    const int wv = (w_lo + lane < w_hi) ? arr[w_lo + lane] : 0x7fffffff;
                    s_win[lane] = wv;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    if (mine) {
                        int lo = 0, hi = w_hi - w_lo;
                        while (lo < hi) { const int mid = (lo + hi) >> 1; if (s_win[mid] < my_tok) lo = mid + 1; else hi = mid; }
                        if (lo < w_hi - w_lo && s_win[lo] == my_tok) found = w_lo + lo;
                    }
                    __builtin_amdgcn_wave_barrier();
                } else if (mine) {
                    const int f = find_sorted(arr + w_lo, w_hi - w_lo, my_tok);
                    found = (f >= 0) ? w_lo + f : -1;
                }
                if (mine) {
                    if (side == 0) my_vslot = found;            // K item: FP16 V row if the token is a V anchor too
                    else if (found >= 0) my_valid = 0;          // V item whose token is also a K anchor: skip
                }
            }
            // 16-byte chunk c (channels 8c .. 8c+7) of an item's effective row: from the FP16 row, or centroids
            // looked up from the token's codes; zero for an entry that is skipped
            auto fetch_chunk = [&](bool valid, int slot, const half_t* rows, int64_t n_rows_per_bg, int tok,
                                   const uint8_t* codes, const half_t* cb, int c) -> uint4_t {
                uint4_t r = {0u, 0u, 0u, 0u};
                if (valid) {
                    if (slot >= 0) {
                        r = *(const uint4_t*)(rows + ((int64_t)bg * n_rows_per_bg + slot) * kD + 8 * c);
                    } else if constexpr (DSUB == 8) {
                        const uint32_t code = codes[(int64_t)tok * M + c];
                        r = *(const uint4_t*)(cb + ((int64_t)c * 256 + code) * 8);
                    } else if constexpr (DSUB == 16) {
                        const int m = c >> 1;
                        const uint32_t code = codes[(int64_t)tok * M + m];
                        r = *(const uint4_t*)(cb + ((int64_t)m * 256 + code) * 16 + 8 * (c & 1));
                    } else {
                        const uint32_t c0 = codes[(int64_t)tok * M + 2 * c], c1 = codes[(int64_t)tok * M + 2 * c + 1];
                        const uint2_t lo = *(const uint2_t*)(cb + ((int64_t)(2 * c) * 256 + c0) * 4);
                        const uint2_t hi = *(const uint2_t*)(cb + ((int64_t)(2 * c + 1) * 256 + c1) * 4);
                        r = uint4_t{lo[0], lo[1], hi[0], hi[1]};
                    }
                }
                return r;
            };
            // ---- scores: S[head][item] for the two 16-item halves.  The dense operand (item along n, channels
            // along k) is 8 consecutive channels per lane: it comes straight from global memory.
            uint4_t kb[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int i_tok = __shfl(my_tok, 16 * u + arow, 64), i_slot = __shfl(my_kslot, 16 * u + arow, 64);
                const bool i_valid = __shfl(my_valid, 16 * u + arow, 64) != 0;
#pragma unroll
                for (int st = 0; st < 4; ++st)
                    kb[u][st] = fetch_chunk(i_valid, i_slot, p.rows_k, p.k_k, i_tok, ck, cbk, 4 * st + kgrp);
            }
            // V rows go through LDS for the transposed reads, 8 items x 64 channels at a time (two of the four
            // transposed reads of one sparse MFMA): for MFMA i, element-quad pair eh and slab set a this lane
            // supplies chunk 8a + lane % 8 of item 16 i + 4 (lane / 16) + 2 eh + (lane / 8) % 2
            uint4_t vq[2][2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int eh = 0; eh < 2; ++eh) {
                    const int it = 16 * i + 4 * kgrp + 2 * eh + ((lane >> 3) & 1);
                    const int r_tok = __shfl(my_tok, it, 64), r_vslot = __shfl(my_vslot, it, 64);
                    const bool r_valid = __shfl(my_valid, it, 64) != 0;
#pragma unroll
                    for (int a = 0; a < 2; ++a)
                        vq[i][eh][a] = fetch_chunk(r_valid, r_vslot, p.rows_v, p.k_v, r_tok, cv, cbv, 8 * a + (lane & 7));
                }
            float sc[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float4_t c4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    half8_t qa = *(const half8_t*)(s_qh + (arow & 3) * kD + 32 * st + 8 * kgrp);
                    if (arow >= kNH) qa = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
                    c4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa, __builtin_bit_cast(half8_t, kb[u][st]), c4, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[u][r] = c4[r] * p.c1;   // lanes 0..15: head r, item 16u + lane
            }
            float mx[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) mx[h] = kNegBig;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bool valid = __shfl(my_valid, 16 * u + arow, 64) != 0;
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
                acc[0][0][h] *= alpha;
                acc[1][0][h] *= alpha;
                m_ref[h] = m_new;
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pw = fast_exp2(sc[u][r] - m_ref[r]);       // 0 for masked / non-row lanes
                    l_lane[r] += pw;
                    if (kgrp == 0) s_p[r * kPStride + p_slot(u, arow >> 2, arow & 3)] = (half_t)pw;
                }
            // ---- P.V: (item, slab) pairs along k; transposed LDS reads turn row-major V rows into the dense operand
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const half8_t pa = load_pa(i);
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    half4_t vb[4];
#pragma unroll
                    for (int eh = 0; eh < 2; ++eh) {
                        *(uint4_t*)(s_vrows + (2 * kgrp + ((lane >> 3) & 1)) * 64 + 8 * (lane & 7)) = vq[i][eh][a];
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
#pragma unroll
                        for (int e = 0; e < 2; ++e)
                            vb[2 * eh + e] = lds_read_tr16(lsm, rows_off + (uint32_t)((2 * kgrp + e) * 64 + 16 * tj + 4 * tq) * 2);
                        __builtin_amdgcn_wave_barrier();
                    }
                    const half16_t bop = {vb[0][0], vb[0][1], vb[0][2], vb[0][3], vb[1][0], vb[1][1], vb[1][2], vb[1][3],
                                          vb[2][0], vb[2][1], vb[2][2], vb[2][3], vb[3][0], vb[3][1], vb[3][2], vb[3][3]};
                    acc[a][0] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(pa, bop, acc[a][0], sm_idx, 0, 0);
                }
            }
        }
        // hand the weight sums over in the stream's form: head lane % 4 in each lane (here: all of it in lanes 0..3)
        float tot = 0.f;
#pragma unroll
        for (int h = 0; h < kNH; ++h) {
            const float t = wave_sum(l_lane[h]);
            tot = (lane == h) ? t : tot;
        }
        l_own = tot;
    }

    // ================================================================================== stream
    {
        // Lane roles.  Code loads and the K side: lane L of the wave handles token L of the tile; the token's class
        // is c = L / 16 and its rank r = L % 16.  The int8 MFMA leaves lane (4 c + h, k-group g) with head h's
        // scores of tokens (c, 4 g + i), i = 0..3: from there on a lane works for one head (tq) and one class (tj).
        // K gather: this lane visits sub-space (step XOR xr) mod M at every step and reads slot (step XOR xr)
        const uint32_t xr = lane & 31;
        const uint32_t kr = xr & (M - 1);                            // XOR applied to the code byte index
        static_assert(L::lut == 0, "the table gather address is an absolute LDS address below 64 KB");
        uint32_t ksel[4], kc[CW];
#pragma unroll
        for (int j = 0; j < 4; ++j) ksel[j] = 0x0c0c0000u | ((4u + (uint32_t)(j ^ (kr & 3))) << 8) | (uint32_t)j;
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            kc[i] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) kc[i] |= ((xr ^ (uint32_t)(4 * i + j)) << 3) << (8 * j);
        }
        // constant operand of the int8 MFMA: column 4 g + h takes, from k-group g only, the (lo, hi) bytes of head h
        // with the weights (1, -128)
        int4_t k_wgt;
        {
            const int col_blk = (lane & 15) >> 2, col_h = lane & 3;
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                uint32_t wv = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = 4 * dw + j;                              // byte of the 16-byte operand
                    const uint32_t wt = (i & 1) ? 0x80u : 0x01u;           // -128 on hi bytes, 1 on lo bytes
                    if (kgrp == col_blk && ((i & 7) >> 1) == col_h) wv |= wt << (8 * j);
                }
                k_wgt[dw] = (int)wv;
            }
        }
        // V gather address = table base | code << 8 | byte offset of the 8-byte piece inside the code's row, the piece
        // being chunk tq of slab 4 a + (tj + rho) % 4 (128 a goes into the instruction's immediate): one byte permute
        // of a staged code dword and a per-lane constant
        static_assert((L::cbv & 0xffff) == 0, "the V table base must be a multiple of 64 KB");
        const uint32_t lds0 = (uint32_t)(uintptr_t)lsm;
        uint32_t v_const[4];
#pragma unroll
        for (int rho = 0; rho < 4; ++rho)
            v_const[rho] = (uint32_t)(32 * ((tj + rho) & 3) + 8 * tq) | (((L::cbv + lds0) >> 16) << 16);
        // The writer (lane = token) rotates its code bytes by its class, so that the byte of slab (c + rho) % 4 sits
        // at the place of slab rho: the reader's byte position then depends on rho (and its chunk) only.
        //   d = 8:  per half (8 bytes) the byte pairs rotate; byte of (rho, chunk) = dword rho / 2, byte 2 (rho % 2) + tq / 2
        //   d = 16: per half (4 bytes) the bytes rotate;      byte of rho          = byte rho of dword a
        //   d = 4:  per half (16 bytes) the dwords rotate;    byte of (rho, chunk) = dword rho, byte tq
        uint32_t v_sel[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t byte = (DSUB == 8) ? (uint32_t)(2 * u + (tq >> 1)) : (uint32_t)tq;
            v_sel[u] = 0x0c020000u | ((4u + byte) << 8);
        }
        uint32_t rot_lo = 0, rot_hi = 0;                             // d = 8: byte selectors of the rotated half
        if constexpr (DSUB == 8) {
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                rot_lo |= (uint32_t)(2 * ((kgrp + (bb >> 1)) & 3) + (bb & 1)) << (8 * bb);
                rot_hi |= (uint32_t)(2 * ((kgrp + 2 + (bb >> 1)) & 3) + (bb & 1)) << (8 * bb);
            }
        }
        // staging: token (c, r) lives in unit 16 c + (r XOR 4 c) (16-byte units, 8-byte for d = 16): writes of a class
        // and reads of a rank both spread over all banks
        constexpr int SU = (DSUB == 16) ? 8 : 16;
        const uint32_t stg0 = lds0 + (uint32_t)(L::pst + wave * kStgBytes);
        const uint32_t stg_w = stg0 + (uint32_t)SU * (uint32_t)(16 * kgrp + ((lane & 15) ^ (4 * kgrp)));
        // reader (k-group kgrp, class tj): element quad e4 holds the token of rank 8 (e4 / 2) + 4 (kgrp / 2) + 2 (kgrp % 2) + e4 % 2
        const uint32_t rb = (uint32_t)((4 * (kgrp >> 1) + 2 * (kgrp & 1)) ^ (4 * tj));
        const uint32_t stg_r0 = stg0 + (uint32_t)SU * (uint32_t)(16 * tj + rb);          // e4 = 0 (and 1 at + SU)
        const uint32_t stg_r1 = stg0 + (uint32_t)SU * (uint32_t)(16 * tj + (rb ^ 8));    // e4 = 2 (and 3 at + SU)
        // anchored-token bits of this lane's four tokens: bits 16 tj + 4 kgrp + i of the tile's 64-bit mask
        const uint32_t mask_dw = (uint32_t)(tj >> 1);
        const uint32_t mask_sh = (uint32_t)(16 * (tj & 1) + 4 * kgrp);

        const int64_t n_tiles = (t1 - t0 + 63) >> 6;
        auto grab_tile = [&]() -> int64_t {
            int t = 0;
            if (lane == 0) t = atomicAdd(&s_misc[8], 1);
            return (int64_t)__builtin_amdgcn_readfirstlane(t);
        };
        // code loads run one tile ahead of their use: HBM latency hides behind the previous tile's work
        auto load_codes = [&](int64_t tile, uint32_t (&kw_)[CW], uint32_t (&vw_)[CW]) {
            const int64_t tok_ = t0 + tile * 64 + lane;
            const int64_t ltok = (tok_ < p.N) ? tok_ : (p.N - 1);        // tokens past the range are masked, not skipped
            if (CW == 2) {
                const uint2_t a = *(const uint2_t*)(ck + ltok * M), c = *(const uint2_t*)(cv + ltok * M);
                kw_[0] = a[0]; kw_[1] = a[1]; vw_[0] = c[0]; vw_[1] = c[1];
            } else {
#pragma unroll
                for (int i = 0; i < CW / 4; ++i) {
                    const uint4_t a = *(const uint4_t*)(ck + ltok * M + 16 * i), c = *(const uint4_t*)(cv + ltok * M + 16 * i);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { kw_[4 * i + e] = a[e]; vw_[4 * i + e] = c[e]; }
                }
            }
        };
        // this lane's head: table quantum and running reference
        float lut_q = ((const float*)s_misc)[12], neg_m = -m_ref[0];
#pragma unroll
        for (int h = 1; h < kNH; ++h) {
            lut_q = (tq == h) ? ((const float*)s_misc)[12 + h] : lut_q;
            neg_m = (tq == h) ? -m_ref[h] : neg_m;
        }

        auto do_tile = [&](int64_t tile, const uint32_t (&kw_in)[CW], const uint32_t (&vw)[CW]) {
            // ---- V code bytes into the staging area (first round; d = 4 stages its second half later)
            if constexpr (DSUB == 8) {
                uint4_t w4;
                w4[0] = __builtin_amdgcn_perm(vw[1], vw[0], rot_lo); w4[1] = __builtin_amdgcn_perm(vw[1], vw[0], rot_hi);
                w4[2] = __builtin_amdgcn_perm(vw[3], vw[2], rot_lo); w4[3] = __builtin_amdgcn_perm(vw[3], vw[2], rot_hi);
                *(__attribute__((address_space(3))) uint4_t*)(uintptr_t)stg_w = w4;
            } else if constexpr (DSUB == 16) {
                uint2_t w2;
                w2[0] = __builtin_amdgcn_alignbit(vw[0], vw[0], 8u * (uint32_t)kgrp);
                w2[1] = __builtin_amdgcn_alignbit(vw[1], vw[1], 8u * (uint32_t)kgrp);
                *(__attribute__((address_space(3))) uint2_t*)(uintptr_t)stg_w = w2;
            }
            auto stage_d4 = [&](int a) {
                uint32_t t[4];
                uint4_t w4;
#pragma unroll
                for (int rho = 0; rho < 4; ++rho) t[rho] = (kgrp & 1) ? vw[4 * a + ((rho + 1) & 3)] : vw[4 * a + rho];
#pragma unroll
                for (int rho = 0; rho < 4; ++rho) w4[rho] = (kgrp & 2) ? t[(rho + 2) & 3] : t[rho];
                *(__attribute__((address_space(3))) uint4_t*)(uintptr_t)stg_w = w4;
            };
            if constexpr (DSUB == 4) stage_d4(0);
            const uint32_t mw = s_mask[(2 * (uint32_t)tile + mask_dw) & (L::mask_words - 1)];

            // ---- K side: scores in log2 units.  Code dwords are XOR-permuted so that step s finds the code of
            // sub-space (s XOR kr) at a compile-time register and a per-lane constant byte selector.
            uint32_t kw[CW];
#pragma unroll
            for (int i = 0; i < CW; ++i) kw[i] = kw_in[i];
#pragma unroll
            for (int bit = 0; (4 << bit) < M; ++bit) {
                const bool sw = (kr >> (2 + bit)) & 1u;
#pragma unroll
                for (int i = 0; i < CW; ++i) {
                    if (!(i & (1 << bit))) {
                        const uint32_t a = kw[i], c = kw[i | (1 << bit)];
                        kw[i] = sw ? c : a;
                        kw[i | (1 << bit)] = sw ? a : c;
                    }
                }
            }
            // One table read per (token, sub-space): the address (code << 8 | slot << 3) is a single byte permute
            // of the code dword and a per-lane constant.  Two entries (16 bytes) are this lane's row of the int8
            // MFMA's first operand (row = rank, k-group = class); the constant second operand routes them.
            // (all gathers of a batch of 16 sub-spaces are issued before the first of them is waited for: with four
            // waves per SIMD a chain of gather -> wait -> MFMA steps leaves the LDS latency exposed)
            int4_t si = {0, 0, 0, 0};
            constexpr int KB = M < 16 ? M : 16;
#pragma unroll
            for (int s0 = 0; s0 < M; s0 += KB) {
                uint2_t ent[KB];
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int st = s0 + u;
                    ent[u] = *(const lds_uint2*)(uintptr_t)__builtin_amdgcn_perm(kw[st >> 2], kc[st >> 2], ksel[st & 3]);
                }
#pragma unroll
                for (int u = 0; u < KB; u += 2)
                    si = __builtin_amdgcn_mfma_i32_16x16x64_i8(int4_t{(int)ent[u][0], (int)ent[u][1], (int)ent[u + 1][0], (int)ent[u + 1][1]},
                                                               k_wgt, si, 0, 0, 0);
            }
            // ---- softmax: register i = token (tj, 4 kgrp + i), head tq.  x = score - reference.
            const uint32_t keep_bits = ~mw >> mask_sh;                 // bit i set: token i is neither anchored nor past the range
            float x[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = fmaf((float)si[i], lut_q, neg_m);
            if (__any(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])) > kPShift)) {
                // some score exceeds the running maximum by more than the head room: move the reference, rescale
                float lm = kNegBig;
#pragma unroll
                for (int i = 0; i < 4; ++i) lm = fmaxf(lm, ((keep_bits >> i) & 1u) ? x[i] : kNegBig);
                lm = fmaxf(lm, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, lm), 0x124, 0xf, 0xf, true)));   // row_ror:4
                lm = fmaxf(lm, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, lm), 0x128, 0xf, 0xf, true)));   // row_ror:8
                lm = fmaxf(lm, __shfl_xor(lm, 16, 64));
                lm = fmaxf(lm, __shfl_xor(lm, 32, 64));                // largest unmasked x of head tq in the tile
                const float m_old = -neg_m;
                const float m_new = fmaxf(m_old, (lm - neg_m) - kPShift);
                const float alpha = fast_exp2(m_old - m_new);
                l_own *= alpha;
                neg_m = -m_new;
                // (multiplied in place through inline assembly: written as plain C++ the compiler keeps a second copy
                // of the 32 accumulator registers for this rare path and moves all of them on every tile)
#pragma unroll
                for (int h = 0; h < kNH; ++h) {
                    const float ah = lane_bcast(alpha, h);              // lanes 0..3 work for heads 0..3
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int rho = 0; rho < 4; ++rho) {
                            float v = acc[a][rho][h];
                            asm volatile("v_mul_f32 %0, %1, %0" : "+v"(v) : "s"(ah));
                            acc[a][rho][h] = v;
                        }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = fmaf((float)si[i], lut_q, neg_m);
            }
            uint4_t pa4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t keep;                                           // all ones or zero (the compiler would turn the
                asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(keep) : "v"(keep_bits), "n"(i));   // builtin into test + select)
                const float pw = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, fast_exp2(x[i])) & keep);
                l_own += pw;
                pa4[i] = (uint32_t)__builtin_bit_cast(unsigned short, (half_t)pw);
            }
            const half8_t pa = __builtin_bit_cast(half8_t, pa4);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();

            // ---- V side: MFMA (a, rho): element quad e4 of this lane's k-group = token (tj, rank(e4)) with slab
            // 4 a + (tj + rho) % 4, the four rows of a transposed read being the four classes
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                constexpr int VD = (DSUB == 4) ? 4 : 2;                // staged code dwords per token and read
                uint32_t vt[4][VD];
                if (a == 0 || DSUB != 16) {
                    if constexpr (DSUB == 4) {
                        if (a == 1) {
                            __builtin_amdgcn_wave_barrier();
                            stage_d4(1);
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                            __builtin_amdgcn_wave_barrier();
                        }
                    }
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const uint32_t ad = ((e4 >> 1) ? stg_r1 : stg_r0) + (uint32_t)(SU * (e4 & 1)) + (DSUB == 8 ? 8u * a : 0u);
                        if constexpr (DSUB == 4) {
                            const uint4_t r = *(const __attribute__((address_space(3))) uint4_t*)(uintptr_t)ad;
#pragma unroll
                            for (int u = 0; u < 4; ++u) vt[e4][u] = r[u];
                        } else {
                            const uint2_t r = *(const lds_uint2*)(uintptr_t)ad;
                            vt[e4][0] = r[0]; vt[e4][1] = r[1];
                        }
                    }
                }
                auto fetch = [&](int rho, half4_t (&vb)[4]) {
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        uint32_t ad;
                        if constexpr (DSUB == 8) ad = __builtin_amdgcn_perm(vt[e4][rho >> 1], v_const[rho], v_sel[rho & 1]);
                        else if constexpr (DSUB == 16) ad = __builtin_amdgcn_perm(vt[e4][a], v_const[rho], 0x0c020000u | ((4u + (uint32_t)rho) << 8));
                        else ad = __builtin_amdgcn_perm(vt[e4][rho], v_const[rho], v_sel[0]);
                        vb[e4] = lds_read_tr16_abs(ad + 128 * a);
                    }
                };
                half4_t vb0[4], vb1[4];
                fetch(0, vb0);
#pragma unroll
                for (int rho = 0; rho < 4; ++rho) {
                    half4_t (&cur)[4] = (rho & 1) ? vb1 : vb0;
                    half4_t (&nxt)[4] = (rho & 1) ? vb0 : vb1;
                    if (rho + 1 < 4) fetch(rho + 1, nxt);
                    const half16_t bop = {cur[0][0], cur[0][1], cur[0][2], cur[0][3], cur[1][0], cur[1][1], cur[1][2], cur[1][3],
                                          cur[2][0], cur[2][1], cur[2][2], cur[2][3], cur[3][0], cur[3][1], cur[3][2], cur[3][3]};
                    acc[a][rho] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(pa, bop, acc[a][rho], sm_idx, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        };

        // The next tile's codes are requested before the current tile is worked on.  The request is unconditional (a
        // wave that has no further tile re-reads the range's last one): a conditional load would cost register copies
        // on every tile.
        uint32_t kw_next[CW], vw_next[CW];
        int64_t tile = grab_tile();
        load_codes(tile < n_tiles ? tile : n_tiles - 1, kw_next, vw_next);
        while (tile < n_tiles) {
            uint32_t kw_c[CW], vw_c[CW];
#pragma unroll
            for (int i = 0; i < CW; ++i) { kw_c[i] = kw_next[i]; vw_c[i] = vw_next[i]; }
            const int64_t tile_next = grab_tile();
            load_codes(tile_next < n_tiles ? tile_next : n_tiles - 1, kw_next, vw_next);
            do_tile(tile, kw_c, vw_c);
            tile = tile_next;
        }
#pragma unroll
        for (int h = 0; h < kNH; ++h) m_ref[h] = -lane_bcast(neg_m, h);
    }
    // weight sums per head: add up the lanes that worked for the head
    float l_sum[kNH];
    {
        float v = l_own;
        v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x124, 0xf, 0xf, true));   // row_ror:4
        v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x128, 0xf, 0xf, true));   // row_ror:8
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
#pragma unroll
        for (int h = 0; h < kNH; ++h) l_sum[h] = lane_bcast(v, h);
    }
    wg_merge_and_store<DSUB>(smem, m_ref, l_sum, acc, part_bg, sp, p.S, nheads);
    // The last workgroup of this (sequence, KV head) to arrive merges the S partials by log-sum-exp and
    // rounds once to fp16: out = sum_s acc_s 2^(m_s - m) / sum_s l_s 2^(m_s - m).
    // Ordering without a cache-wide release: the partial was written with device-scope stores, each wave
    // waits for its own stores to be acknowledged, the barrier collects the waves, and only then does one
    // thread bump the device-scope counter.  The merging workgroup reads with device-scope loads.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0)
        s_misc[10] = (int)(unsigned int)__hip_atomic_fetch_add(&p.done[bg], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
    __syncthreads();
    if (s_misc[10] == p.S) {
        // S can be a few hundred: the statistics of all slots go through LDS first (one round of loads), then every
        // (head, channel) thread sums its column with eight independent loads in flight.
        auto ld = [](const float* q) { return __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
        float* s_w = (float*)(smem + L::mrg);                       // [4 heads][S]: slot weights 2^(m_s - m) (table area is free now)
        float* s_tot = s_w + kNH * 1024;                            // [4]: total l per head
        const int S = p.S;
        for (int i = tid; i < kNH * S; i += kDaThreads) {
            const int h = i / S, sl = i - h * S;
            s_w[h * 1024 + sl] = (h < nheads) ? ld(part_bg + ((int64_t)h * S + sl) * (kD + 2) + kD) : kNegBig;
        }
        __syncthreads();
        if (wave < kNH) {                                           // one wave per head: global maximum, weights, total
            const int h = wave;
            float m = kNegBig;
            for (int sl = lane; sl < S; sl += 64) m = fmaxf(m, s_w[h * 1024 + sl]);
            m = wave_max(m);
            float l = 0.f;
            for (int sl = lane; sl < S; sl += 64) {
                const float w = fast_exp2(s_w[h * 1024 + sl] - m);
                s_w[h * 1024 + sl] = w;
                if (h < nheads) l += ld(part_bg + ((int64_t)h * S + sl) * (kD + 2) + kD + 1) * w;
            }
            l = wave_sum(l);
            if (lane == 0) s_tot[h] = l;
        }
        __syncthreads();
        if (tid < kNH * kD) {
            const int h = tid >> 7, dim = tid & 127;
            if (h < nheads) {
                const float* pb = part_bg + (int64_t)h * S * (kD + 2) + dim;
                float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                int sl = 0;
                for (; sl + 8 <= S; sl += 8) {
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = ld(pb + (int64_t)(sl + u) * (kD + 2));
#pragma unroll
                    for (int u = 0; u < 8; ++u) a8[u] = fmaf(v[u], s_w[h * 1024 + sl + u], a8[u]);
                }
                for (; sl < S; ++sl) a8[0] = fmaf(ld(pb + (int64_t)sl * (kD + 2)), s_w[h * 1024 + sl], a8[0]);
                const float a = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
                const float l = s_tot[h];
                p.out[((int64_t)b * p.Hq + h0 + h) * kD + dim] = (half_t)(l > 0.f ? a / l : 0.f);
            }
        }
    }
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
    float *ans_k, *ans_v;  // [B][Hkv][N]
    int64_t N, N_cap;
    int k_k;
    float c1;
    int Hq, Hkv, G, S;
    int64_t chunk;
    uint32_t* hist;             // optional (pass 1): first-level top-k histograms, [2 B Hkv][2 * kTopkBins], K rows then V rows
};

template <int DSUB, int PASS>
__global__ __launch_bounds__(kDaThreads) void decode_ans_kernel(const DsParams p)
{
    constexpr int M = kD / DSUB;
    constexpr int CW = M / 4;
    // The table is code-major, [256 codes][SLOTS] entries of 4 heads x fp32 (16 bytes), slot s holding sub-space s mod M:
    // the bank group of an entry (slot mod 16) then depends on the slot alone, and the 16 lanes of an LDS pass, which
    // visit sub-space (step XOR lane) in copy (lane / M), hit 16 different groups whatever the codes are.
    constexpr int SLOTS = M < 16 ? 16 : M;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    float4_t* s_lut = (float4_t*)smem;                      // [256][SLOTS] x 4 heads fp32
    float* s_qf = (float*)(smem + SLOTS * 256 * 16);        // [4][128]
    float* s_red = s_qf + kNH * kD;                         // [waves][8]
    int* s_misc = (int*)(s_red + kDaWaves * 8);             // 16 ints
    uint32_t* s_mask = (uint32_t*)(s_misc + 16);            // bitmap of K-anchored tokens, 1024 words
    uint32_t* s_hist = s_mask + 1024;                       // pass 1 with p.hist: [2][kTopkBins] counts of the scores written
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bg = blockIdx.x / p.S, sp = blockIdx.x % p.S;
    const int b = bg / p.Hkv, g = bg % p.Hkv;
    const int h0 = g * p.G;
    const half_t* qb = p.q + ((int64_t)b * p.Hq + h0) * kD;
    const int32_t* idx_k = p.idx_k + (int64_t)bg * p.k_k;
    const int64_t t0 = (int64_t)sp * p.chunk;
    const int64_t t1 = (t0 + p.chunk < p.N) ? t0 + p.chunk : p.N;

    // K-anchored tokens are scored from their FP16 rows after the code stream, 16 lanes per token and 8 channels each;
    // blocks of 64 list entries are dealt round-robin over the S workgroups of the (sequence, KV head), whatever token
    // range an entry falls into, so that anchors clustered in one part of the context do not pile up in one
    // workgroup.  The loads of a wave's first kPre rounds are issued here, ahead of everything else: one after the
    // other behind the stream they were a chain of exposed load latencies.
    constexpr int kPre = 4;
    const int a_sub = lane >> 4, a_l16 = lane & 15;
    const int a_first = sp * (4 * kDaWaves) + 4 * wave, a_stride = p.S * (4 * kDaWaves);
    int pre_tok[kPre];
    half8_t pre_v[kPre];
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int i = a_first + u * a_stride + a_sub;
        const bool on = i < p.k_k;
        pre_tok[u] = -1;
        pre_v[u] = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (on) {     // an empty K list may come with null pointers: nothing is read then
            pre_tok[u] = idx_k[i];
            pre_v[u] = *(const half8_t*)(p.rows_k + ((int64_t)bg * p.k_k + i) * kD + 8 * a_l16);
        }
    }
    // this thread's centroids (entries tid + 1024 j of the table): loaded before the barrier, used after it
    constexpr int kEnt = M * 256 / kDaThreads;
    const half_t* cbk = p.cb_k + (size_t)g * 32768;
    uint4_t cen[kEnt][(DSUB + 7) / 8];
#pragma unroll
    for (int j = 0; j < kEnt; ++j) {
        const int e = tid + j * kDaThreads;
        if constexpr (DSUB == 4) {
            const uint2_t v = *(const uint2_t*)(cbk + e * 4);
            cen[j][0] = uint4_t{v[0], v[1], 0u, 0u};
        } else {
#pragma unroll
            for (int u = 0; u < DSUB / 8; ++u) cen[j][u] = *(const uint4_t*)(cbk + e * DSUB + 8 * u);
        }
    }
    if (tid < kNH * kD) s_qf[tid] = ((tid >> 7) < p.G) ? (float)qb[tid] : 0.f;
    for (int i = tid; i < 1024; i += kDaThreads) s_mask[i] = 0u;
    const bool count_scores = PASS == 1 && p.hist != nullptr;
    if (count_scores)
        for (int i = tid; i < 2 * kTopkBins; i += kDaThreads) s_hist[i] = 0u;
    // K-anchored positions of this range: a list of up to 16 K entries is scanned whole (independent loads, one load
    // latency); a longer one is cut to the range by a cooperative search first (a few dependent load latencies)
    const bool scan_list = p.k_k <= 16 * kDaThreads;
    if (!scan_list && wave < 2) {
        const int r = wave_lower_bound(idx_k, p.k_k, (int)(wave ? t1 : t0), lane);
        if (lane == 0) s_misc[wave] = r;
    }
    __syncthreads();
    {
        // fp32 table: entry e = (m, code) holds the four heads' c1 * q_h[m] . cb_k[g][m][code]
#pragma unroll
        for (int j = 0; j < kEnt; ++j) {
            const int e = tid + j * kDaThreads;
            const int m = e >> 8;
            float cf[DSUB];
#pragma unroll
            for (int u = 0; u < (DSUB + 7) / 8; ++u) {
                const half8_t v = __builtin_bit_cast(half8_t, cen[j][u]);
#pragma unroll
                for (int t = 0; t < (DSUB < 8 ? DSUB : 8); ++t) cf[8 * u + t] = (float)v[t];
            }
            float4_t o;
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                float s = 0.f;
#pragma unroll
                for (int t = 0; t < DSUB; ++t) s = fmaf(s_qf[h * kD + m * DSUB + t], cf[t], s);
                o[h] = s * p.c1;
            }
#pragma unroll
            for (int c = 0; c < SLOTS / M; ++c) s_lut[(e & 255) * SLOTS + m + M * c] = o;
        }
    }
    if (scan_list) {
        const uint32_t range_len = (uint32_t)(t1 - t0);
        for (int i0 = tid; i0 < p.k_k; i0 += 4 * kDaThreads) {
            int v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = (i0 + u * kDaThreads < p.k_k) ? idx_k[i0 + u * kDaThreads] : -1;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t rel = (uint32_t)v[u] - (uint32_t)t0;   // positions below t0 (and the -1 filler) wrap to huge values
                if (v[u] >= 0 && rel < range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
    } else {
        for (int i = s_misc[0] + tid; i < s_misc[1]; i += kDaThreads) {
            const int rel = idx_k[i] - (int)t0;
            atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
        }
    }
    // ||q_h||_2: one wave per head
    if (wave < kNH) {
        const float a = s_qf[wave * kD + lane], c = s_qf[wave * kD + 64 + lane];
        const float ss = wave_sum(fmaf(a, a, c * c));
        if (lane == 0) s_red[kDaWaves * 8 - 4 + wave] = sqrtf(ss);       // parked in the last wave's slots until the barrier
    }
    // pass 1: log-sum-exp of each head from the S partial (max, sum) pairs that pass 0 left; one wave per head, the
    // lanes share the S pairs
    if (PASS == 1 && wave >= kNH && wave < 2 * kNH) {
        const int h = wave - kNH;
        float v = 0.f;
        if (h < p.G) {
            const float2* sp_ = (const float2*)(p.stat_part + ((int64_t)b * p.Hq + h0 + h) * p.S * 2);
            float m = kNegBig, l = 0.f;                          // per-lane (reference, sum) over its share of the pairs
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
        if (lane == 0) s_red[kDaWaves * 8 - 8 + h] = v;
    }
    __syncthreads();
    float qn[kNH], lse[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) {
        qn[h] = s_red[kDaWaves * 8 - 4 + h];
        lse[h] = (PASS == 1) ? s_red[kDaWaves * 8 - 8 + h] : 0.f;
    }
    __syncthreads();
    const uint8_t* ck = p.codes_k + (int64_t)bg * p.N_cap * M;
    float m_run[kNH], l_run[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) { m_run[h] = kNegBig; l_run[h] = 0.f; }

    // PASS 0 keeps, per lane and head, a sum of exp2(score - reference); the reference only moves when a score
    // exceeds it by more than 64 (or on the lane's first token), so the common token costs one exp2 per head.
    auto consume = [&](const float (&s)[kNH], int64_t tok) {
        if (PASS == 0) {
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float x = s[h] - m_run[h];
                if (x > 64.f) {                                  // first token (reference = kNegBig) or a big jump
                    l_run[h] = l_run[h] * fast_exp2(-x) + 1.f;
                    m_run[h] = s[h];
                } else {
                    l_run[h] += fast_exp2(x);
                }
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
            if (count_scores) {                                  // the selection that follows starts from these counts
                atomicAdd(&s_hist[float_key(ak) >> 21], 1u);
                atomicAdd(&s_hist[kTopkBins + (float_key(av) >> 21)], 1u);
            }
        }
    };

    // ---- code stream: one token per lane, code loads one round ahead; tokens with an FP16 K row are left to
    // the loop below
    auto load_kw = [&](int64_t tok, uint32_t (&kw)[CW]) {
        if (CW == 2) { const uint2_t a = *(const uint2_t*)(ck + tok * M); kw[0] = a[0]; kw[1] = a[1]; }
        else {
#pragma unroll
            for (int i = 0; i < CW / 4; ++i) {
                const uint4_t a = *(const uint4_t*)(ck + tok * M + 16 * i);
#pragma unroll
                for (int e = 0; e < 4; ++e) kw[4 * i + e] = a[e];
            }
        }
    };
    // lane constants of the conflict-free walk: at step st the lane reads sub-space st ^ r
    const int r = lane & (M - 1);
    const uint32_t slot0 = (uint32_t)(r + (M < 16 ? M * ((lane / M) & (16 / M - 1)) : 0)) * 16u;   // byte offset of the slot at step 0
    uint32_t sh4[4];                                              // bit offset of the code byte for step st: sh4[st & 3]
#pragma unroll
    for (int e = 0; e < 4; ++e) sh4[e] = 8u * (uint32_t)(e ^ (r & 3));
    const char* lut_bytes = (const char*)s_lut;
    // code loads run kAhead rounds ahead of their use (more than one round in flight did not pay)
    constexpr int kAhead = 1;
    uint32_t kw_q[kAhead][CW];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
#pragma unroll
        for (int i = 0; i < CW; ++i) kw_q[u][i] = 0u;
        if (t0 + tid + (int64_t)u * kDaThreads < t1) load_kw(t0 + tid + (int64_t)u * kDaThreads, kw_q[u]);
    }
    for (int64_t tok0 = t0 + tid; tok0 < t1; tok0 += (int64_t)kAhead * kDaThreads) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int64_t tok = tok0 + (int64_t)u * kDaThreads;
            uint32_t kw[CW];
#pragma unroll
            for (int i = 0; i < CW; ++i) kw[i] = kw_q[u][i];
            if (tok + (int64_t)kAhead * kDaThreads < t1) load_kw(tok + (int64_t)kAhead * kDaThreads, kw_q[u]);
            if (tok >= t1) continue;
            // code dwords XOR-permuted by r / 4, so that step st finds its dword at the compile-time index st / 4
#pragma unroll
            for (int bit = 0; (4 << bit) < M; ++bit) {
                const bool sw = (r >> (2 + bit)) & 1;
#pragma unroll
                for (int i = 0; i < CW; ++i) {
                    if (!(i & (1 << bit))) {
                        const uint32_t a = kw[i], c = kw[i | (1 << bit)];
                        kw[i] = sw ? c : a;
                        kw[i | (1 << bit)] = sw ? a : c;
                    }
                }
            }
            float s[kNH] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < M; ++st) {
                const uint32_t code = __builtin_amdgcn_ubfe(kw[st >> 2], sh4[st & 3], 8u);
                const uint32_t off = (code * (uint32_t)(SLOTS * 16)) | (slot0 ^ (uint32_t)(16 * st));
                const float4_t e = *(const float4_t*)(lut_bytes + off);
#pragma unroll
                for (int h = 0; h < kNH; ++h) s[h] += e[h];
            }
            const int rel = (int)(tok - t0);
            if (!((s_mask[rel >> 5] >> (rel & 31)) & 1u)) consume(s, tok);
        }
    }
    // ---- K-anchored tokens: the prefetched rounds, then any further ones
    {
        const int l16 = a_l16;
        float qv[kNH][8];
#pragma unroll
        for (int h = 0; h < kNH; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[h][e] = s_qf[h * kD + 8 * l16 + e];
        auto score_row = [&](const half8_t& v, int tok) {
            float s[kNH];
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(qv[h][e], (float)v[e], d);
                s[h] = row16_sum(d) * p.c1;
            }
            if (tok >= 0 && l16 == 0) consume(s, tok);
        };
#pragma unroll
        for (int u = 0; u < kPre; ++u)
            if (a_first + u * a_stride < p.k_k) score_row(pre_v[u], pre_tok[u]);        // uniform per wave
        for (int i0 = a_first + kPre * a_stride; i0 < p.k_k; i0 += a_stride) {
            const int i = i0 + a_sub;
            const bool on = i < p.k_k;
            const int tok = on ? idx_k[i] : -1;
            const half8_t v = *(const half8_t*)(p.rows_k + ((int64_t)bg * p.k_k + (on ? i : 0)) * kD + 8 * l16);
            score_row(v, tok);
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
    if (count_scores) {
        __syncthreads();
        uint32_t* hk = p.hist + (int64_t)bg * 2 * kTopkBins;
        uint32_t* hv = p.hist + ((int64_t)gridDim.x / p.S + bg) * 2 * kTopkBins;     // V rows follow the B * Hkv K rows
        for (int i = tid; i < kTopkBins; i += kDaThreads) {
            if (s_hist[i]) atomicAdd(&hk[i], s_hist[i]);
            if (s_hist[kTopkBins + i]) atomicAdd(&hv[i], s_hist[kTopkBins + i]);
        }
    }
}


struct DaPlan {
    int S;
    int64_t chunk;
    size_t off_part, off_done, off_stat, total;
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
    (void)k_k; (void)k_v;
    size_t off = 0;
    pl.off_part = off; off += align_up((size_t)g.B * g.Hq * pl.S * (kD + 2) * sizeof(float));
    pl.off_done = off; off += align_up((size_t)g.B * g.Hkv * sizeof(unsigned long long));
    pl.off_stat = off; off += want_ans ? align_up((size_t)g.B * g.Hq * pl.S * 2 * sizeof(float)) : 0;
    pl.total = off;
    return pl;
}

}  // namespace

int decode_num_splits(const Geom& g, int64_t N) { return da_plan(g, N, 0, 0, false).S; }

size_t decode_workspace_bytes(const Geom& g, int64_t N, int64_t k_k, int64_t k_v, bool want_ans)
{
    return da_plan(g, N, k_k, k_v, want_ans).total;
}

// Launch tags are unique within the process (a wrap after 2^32 launches could only matter for a workspace
// last used exactly 2^32 launches earlier); 0 is never handed out.
static unsigned int next_launch_tag()
{
    static std::atomic<unsigned int> counter{1u};
    unsigned int t = counter.fetch_add(1u, std::memory_order_relaxed);
    if (t == 0u) t = counter.fetch_add(1u, std::memory_order_relaxed);
    return t;
}

template <int DSUB>
static hipError_t launch_decode_t(const Geom& g, const DecodeArgs& a, void* ws, hipStream_t st)
{
    const bool want_ans = a.ans_k || a.ans_v;
    const DaPlan pl = da_plan(g, a.N, a.k_k, a.k_v, want_ans);
    char* w = (char*)ws;
    float* part = (float*)(w + pl.off_part);
    DaParams p;
    p.q = a.q; p.codes_k = a.codes_k; p.codes_v = a.codes_v; p.cb_k = a.cb_k; p.cb_v = a.cb_v;
    p.idx_k = a.idx_k; p.idx_v = a.idx_v; p.rows_k = a.rows_k; p.rows_v = a.rows_v;
    p.part = part; p.out = a.out; p.done = (unsigned long long*)(w + pl.off_done); p.tag = next_launch_tag(); p.N = a.N; p.N_cap = a.N_cap; p.k_k = (int)a.k_k; p.k_v = (int)a.k_v;
    p.c1 = a.scale * kLog2e; p.Hq = g.Hq; p.Hkv = g.Hkv; p.G = g.G; p.S = pl.S; p.chunk = pl.chunk;
    if (pl.S > 1024) return hipErrorInvalidValue;        // the in-kernel merge keeps one weight per slot in LDS
    const size_t shmem = Lds<DSUB>::total;
    // One-time set-up per instantiation (and per process): raise the dynamic LDS limit, and make sure the kernel has
    // no static LDS — its table gathers use absolute LDS addresses, which assumes the dynamic block starts at 0.
    static const hipError_t setup = [] {
        hipFuncAttributes attr;
        hipError_t r = hipFuncGetAttributes(&attr, (const void*)decode_attn_kernel<DSUB>);
        if (r != hipSuccess) return r;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidConfiguration;
        return hipFuncSetAttribute((const void*)decode_attn_kernel<DSUB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)Lds<DSUB>::total);
    }();
    hipError_t e = setup;
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((int64_t)g.B * g.Hkv * pl.S);
    hipLaunchKernelGGL(decode_attn_kernel<DSUB>, dim3(grid), dim3(kDaThreads), shmem, st, p);
    if (want_ans) {
        DsParams d;
        d.q = a.q; d.codes_k = a.codes_k; d.cb_k = a.cb_k; d.idx_k = a.idx_k; d.rows_k = a.rows_k;
        d.stat_part = (float*)(w + pl.off_stat); d.ans_k = a.ans_k; d.ans_v = a.ans_v;
        d.N = a.N; d.N_cap = a.N_cap; d.k_k = (int)a.k_k; d.c1 = p.c1; d.Hq = g.Hq; d.Hkv = g.Hkv; d.G = g.G;
        d.S = pl.S; d.chunk = pl.chunk;
        d.hist = a.topk_hist;
        const size_t sh2 = (size_t)(g.M < 16 ? 16 : g.M) * 256 * 16 + kNH * kD * 4 + kDaWaves * 32 + 64 + 4096 + 2 * kTopkBins * 4;
        static const hipError_t ans_setup = [sh2]() {              // once per process and DSUB
            hipError_t e1 = hipFuncSetAttribute((const void*)decode_ans_kernel<DSUB, 0>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh2);
            if (e1 != hipSuccess) return e1;
            return hipFuncSetAttribute((const void*)decode_ans_kernel<DSUB, 1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)sh2);
        }();
        if (ans_setup != hipSuccess) return ans_setup;
        const unsigned grid2 = (unsigned)((int64_t)g.B * g.Hkv * pl.S);
        hipLaunchKernelGGL((decode_ans_kernel<DSUB, 0>), dim3(grid2), dim3(kDaThreads), sh2, st, d);
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
