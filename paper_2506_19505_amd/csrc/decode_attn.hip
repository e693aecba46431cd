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
//  anchors   the (sequence, KV head)'s anchor lists are cut into tiles (16 K entries or 32 V entries) dealt
//            round-robin to the workgroups (balanced by list index, not by position: anchors cluster at the
//            head and tail of a context) and, inside a workgroup, to the waves: every wave works on its tile
//            before any wave streams, so the entries never compete with the stream for the LDS and the issue
//            slots.  A tile's tokens, cross membership (is the token in the other list too?) and code rows are
//            fetched during the prologue, its FP16 rows just before the prologue's last barrier.  K entries
//            are scored on the dense MFMA (rows straight from global memory into the operand), V entries through
//            the lookup table like the stream; the values are packed fp16 dot products, two entries at a time.
//  stream    wave w starts with tile w, then waves pull 64-token tiles from a shared counter, code loads running
//            one tile ahead:
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
// per-wave staging.  Anchor tiles: code rows of the entries, then the weights of 32 pairs of entries.  Stream: the V code
// bytes of a tile (up to 1 KB).  Prologue: all waves' areas together hold the two anchor lists.
constexpr int kStgBytes = 1664;
static_assert(kStgBytes % 16 == 0, "16-byte accesses to the staging areas");
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

// Workgroup barrier that orders LDS traffic only: global loads still in flight stay in flight (__syncthreads would wait
// for every one of them, which turns each barrier of the prologue into a full memory round trip).  Global stores that
// other waves read after the barrier need a wait of their own before it.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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

typedef __attribute__((address_space(3))) int32_t lds_int;
__device__ __forceinline__ int find_sorted_lds(const lds_int* arr, int n, int key)
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
    int32_t* info;              // [B][Hkv][k_k + k_v] cross membership of the anchor entries, filled in the prologue:
                                // K entry: its slot in the V list or -1; V entry: 1 if the token is a K anchor too (skipped), else 0
    unsigned long long* done;   // [B][Hkv] arrival words (launch tag << 32 | count); the last workgroup of a (b, g) merges
    unsigned int tag;           // this launch's tag: words carrying another tag count as zero, so no clearing pass
    int64_t N, N_cap;
    int k_k, k_v;
    float c1;                   // scale * log2(e)
    int Hq, Hkv, G;
    int S;                      // workgroups (token ranges) per (b, g)
    int64_t chunk;              // tokens per range (multiple of 64)
    // Kernels with given scores: codes_k points to the K side's scores in log2 units instead, fp32
    // [B][Hkv][n_pad / 4][4 heads][4 tokens] with n_pad = N rounded up to 64 (a 64-token tile is 64 float4, float4 number
    // 16 tj + 4 kgrp + tq being what lane (tq, tj, kgrp) of the stream needs); cb_k is not used.
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
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

// MODE is the option mask of antkv_set_decode_options, compiled in so that the default kernel carries none of it:
//   bit 0 (fixed order)  every wave walks a fixed sequence of tiles (w, w + 16, ...) instead of pulling them from the
//                        workgroup's counter: the order of all sums is then fixed and the output is the same bit for bit
//                        on every launch (the counter balances the waves better);
//   bit 2 (long lists)   not an option of the caller: set by the launcher for anchor lists of 3073 .. 16384 entries, which
//                        are then held whole in the two table areas during the prologue (shorter lists fit the waves'
//                        staging areas; longer ones are searched in global memory);
//   bit 1 (wide table)   the lookup table carries a second entry per (code, sub-space), the residual of the first in
//                        units of quantum / 32512, in the slots that otherwise hold copies of the first, and every tile
//                        walks the table twice: 30-bit instead of 15-bit entries, for queries whose products with the
//                        centroids leave the range that the 15-bit quantum serves.  d = 4 has no spare slots (its 32
//                        sub-spaces fill the 32 slots of a row) and ignores the bit.
//   bit 3 (given scores) not an option of the caller: the scores of the K side come from p.scores (keys that are rotated to
//                        their position before the product with q have no table); no table is built, the K codes are
//                        not read, the K anchor list is empty and V entries take their token's score from p.scores.
template <int DSUB, int MODE>
__global__ __launch_bounds__(kDaThreads) void decode_attn_kernel(const DaParams p)
{
    constexpr bool DET = (MODE & 1) != 0;
    constexpr bool WIDE = (MODE & 2) != 0 && DSUB != 4;
    constexpr bool LONG = (MODE & 4) != 0;
    constexpr bool GIVEN = (MODE & 8) != 0;
    static_assert(!GIVEN || (MODE & 6) == 0, "given scores go with the plain tables and short-list prologue only");
    constexpr int M = kD / DSUB;
    constexpr int CW = M / 4;                          // code dwords per token
    static_assert(kDaWaves == 16, "the table build gives each of 16 waves 16 of the 256 codes");
    using L = Lds<DSUB>;
    extern __shared__ uint4_t smem_u4[];
    char* smem = (char*)smem_u4;
    const lds_char* lsm = (const lds_char*)smem_u4;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and the compiler may know it
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
    // anchor entries are processed in tiles dealt round-robin over the S workgroups: K tiles of 16 entries, then V tiles of 32
    const int ntk = (p.k_k + 15) >> 4, ntv = (p.k_v + 31) >> 5;
    const int n_atiles = ntk + ntv;
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
    // The first anchor tile of this wave (tile sp + S * wave of the (sequence, KV head)'s tiles): its tokens, their cross
    // membership and their code rows are fetched during the prologue, while the memory system is idle, so that the
    // tile itself is left with a single round trip (the FP16 rows).
    const int T_first = sp + p.S * wave;
    int pre_tok = 0, pre_info = 0;
    uint32_t pre_codes[CW];
#pragma unroll
    for (int i = 0; i < CW; ++i) pre_codes[i] = 0u;
    // (long-list kernels: a wave often has a second tile, sp + S * (wave + 16); the same is fetched for it, so that the
    // second tile too is left with one round trip, its FP16 rows)
    int pre2_tok = 0, pre2_info = 0;
    uint32_t pre2_codes[CW];
#pragma unroll
    for (int i = 0; i < CW; ++i) pre2_codes[i] = 0u;
    uint32_t pre_rows[32];                         // the tile's FP16 rows, in the form the tile works on (requested before the prologue's last barrier)
    // FP16 K rows of the 16 entries from e0 on as MFMA operands: lane (entry arow, k-group kgrp) holds channels
    // 32 st + 8 kgrp .. + 7 in r[4 st .. 4 st + 3]
    auto load_k_rows = [&](int e0, uint32_t (&r)[32]) {
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            uint4_t v = uint4_t{0u, 0u, 0u, 0u};
            if (e0 + arow < p.k_k) v = *(const uint4_t*)(p.rows_k + ((int64_t)bg * p.k_k + e0 + arow) * kD + 8 * (4 * st + kgrp));
#pragma unroll
            for (int i = 0; i < 4; ++i) r[4 * st + i] = v[i];
        }
    };
    // channels 2 lane, 2 lane + 1 of the FP16 V rows of the 32 entries from j0 on (one coalesced 256-byte load per entry;
    // entries past the list repeat the last row and get weight 0)
    auto load_v_rows = [&](int j0, uint32_t (&r)[32]) {
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const int j = j0 + k;
            r[k] = *(const uint32_t*)(p.rows_v + ((int64_t)bg * p.k_v + (j < p.k_v ? j : p.k_v - 1)) * kD + 2 * lane);
        }
    };
    // given scores: the four heads' scores of one token
    float4_t pre_sc = {0.f, 0.f, 0.f, 0.f};
    auto load_score = [&](int tok) -> float4_t {
        const float* sp_ = (const float*)p.codes_k + ((int64_t)bg * ((p.N + 63) & ~63LL) + (int64_t)(tok & ~3)) * 4 + (tok & 3);
        return float4_t{sp_[0], sp_[4], sp_[8], sp_[12]};
    };
    auto load_codes = [&](const uint8_t* src, uint32_t (&dst)[CW]) {
        if constexpr (CW == 2) {
            const uint2_t a = *(const uint2_t*)src;
            dst[0] = a[0]; dst[1] = a[1];
        } else {
#pragma unroll
            for (int i = 0; i < CW / 4; ++i) {
                const uint4_t a = *(const uint4_t*)(src + 16 * i);
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[4 * i + e] = a[e];
            }
        }
    };

    // ================================================================================== prologue
    {
        // all global loads of the prologue are issued before anything waits on them.
        // the small loads go first: the first barrier then waits for them only, and the two 64 KB tables
        // keep streaming in behind it
        half_t qv16 = (half_t)0.f;
        if (tid < kNH * kD && (tid >> 7) < nheads) qv16 = qb[tid];
        // anchored positions of this range: short lists are scanned whole (one load latency), long lists are
        // cut to the range by a cooperative search first (a few dependent load latencies)
        // both lists are short: they go to LDS whole (into the waves' staging areas, which nobody uses before the
        // anchors), and the bitmap and the cross membership of the anchor entries are worked out from there
        // (long-list kernels, chosen by the host from the list lengths: the lists go to the two table areas instead, up
        // to 16384 entries each, in batches of the same three rounds; the tables are written after the barrier that
        // follows the last use of the lists)
        constexpr int kScanBatch = LONG ? 9 : 3;                  // one load per thread and round, all in flight together
        constexpr int kScanMax = LONG ? 16384 : kScanBatch * kDaThreads;
        static_assert(LONG || 2 * kScanMax * 4 <= kDaWaves * kStgBytes, "two whole lists fit the staging areas");
        static_assert(kScanMax * 4 <= 65536, "a whole list fits one table area");
        const bool lists_in_lds = p.k_k <= kScanMax && p.k_v <= kScanMax;
        int scan_val[2][kScanBatch];
        if (lists_in_lds) {
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i) {
                const int j = tid + i * kDaThreads;
                scan_val[0][i] = (j < p.k_k) ? idx_k[j] : -1;
                scan_val[1][i] = (j < p.k_v) ? idx_v[j] : -1;
            }
        }
        if (wave < 4) {
            const int32_t* arr = (wave < 2) ? idx_k : idx_v;
            const int n = (wave < 2) ? p.k_k : p.k_v;
            int r = 0;
            if (!lists_in_lds) r = wave_lower_bound(arr, n, (int)((wave & 1) ? t1 : t0), lane);
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
            if constexpr (GIVEN) {
                opb[j] = uint4_t{0u, 0u, 0u, 0u};
            } else if constexpr (DSUB == 8) {
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
        if (tid < kNH * kD) ((half_t*)(smem + L::qh))[tid] = qv16;
        int32_t* s_lk = (int32_t*)(smem + (LONG ? L::lut : L::pst));
        int32_t* s_lv = LONG ? (int32_t*)(smem + L::cbv) : s_lk + kScanMax;
        if (lists_in_lds) {
#pragma unroll
            for (int i = 0; i < kScanBatch; ++i) {
                const int j = tid + i * kDaThreads;
                if (j < p.k_k) s_lk[j] = scan_val[0][i];
                if (j < p.k_v) s_lv[j] = scan_val[1][i];
            }
            if constexpr (LONG) {
                // the rest of long lists, three rounds in flight at a time
                const int k_max = p.k_k > p.k_v ? p.k_k : p.k_v;
                for (int base = kScanBatch * kDaThreads; base < k_max; base += kScanBatch * kDaThreads) {
#pragma unroll
                    for (int i = 0; i < kScanBatch; ++i) {
                        const int j = base + tid + i * kDaThreads;
                        scan_val[0][i] = (j < p.k_k) ? idx_k[j] : -1;
                        scan_val[1][i] = (j < p.k_v) ? idx_v[j] : -1;
                    }
#pragma unroll
                    for (int i = 0; i < kScanBatch; ++i) {
                        const int j = base + tid + i * kDaThreads;
                        if (j < p.k_k) s_lk[j] = scan_val[0][i];
                        if (j < p.k_v) s_lv[j] = scan_val[1][i];
                    }
                }
            }
        }
        for (int i = tid; i < L::mask_words; i += kDaThreads) s_mask[i] = 0u;
        if (tid == 0) s_misc[8] = kDaWaves;                      // next stream tile to hand out (wave w starts with tile w)
        lds_barrier();
        if (tid == 0 && ((unsigned int)(done_seen >> 32) != p.tag || (unsigned int)done_seen >= (unsigned int)p.S))
            __hip_atomic_compare_exchange_strong(&p.done[bg], &done_seen, (unsigned long long)p.tag << 32, __ATOMIC_RELAXED,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // bitmap of anchored tokens in this range
        const uint32_t range_len = (uint32_t)(t1 - t0);
        if (lists_in_lds) {
            // unsigned compare: positions below t0 wrap to huge values
            for (int j = tid; j < p.k_k; j += kDaThreads) {
                const uint32_t rel = (uint32_t)((const lds_int*)s_lk)[j] - (uint32_t)t0;
                if (rel < range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
            for (int j = tid; j < p.k_v; j += kDaThreads) {
                const uint32_t rel = (uint32_t)((const lds_int*)s_lv)[j] - (uint32_t)t0;
                if (rel < range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        // positions between the end of the range and the end of its last tile count as anchored: the stream skips them
        if (tid < 64) {
            const uint32_t rel = ((range_len - 1u) & ~63u) + (uint32_t)tid;
            if (rel >= range_len) atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
        }
        if (!lists_in_lds) {
            for (int i = s_misc[0] + tid; i < s_misc[1]; i += kDaThreads) {
                const int rel = idx_k[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        if (!lists_in_lds) {
            for (int i = s_misc[2] + tid; i < s_misc[3]; i += kDaThreads) {
                const int rel = idx_v[i] - (int)t0;
                atomicOr(&s_mask[rel >> 5], 1u << (rel & 31));
            }
        }
        // Cross membership of the anchor entries that this workgroup will process (tiles sp, sp + S, ... of the
        // (sequence, KV head)'s entries: K tiles of 16, then V tiles of 32): a K entry needs to know whether its token
        // has an FP16 V row too (and where), a V entry whether its token is a K anchor (then the K entry covers it).
        {
            // a wave's first tile: one lane per entry, answers stay in registers; the entry's code row is requested at once
            auto resolve_tile = [&](int T, int& tok_o, int& info_o, uint32_t (&codes_o)[CW]) {
                if (T >= n_atiles) return;
                if (T < ntk) {
                    const int e = 16 * T + lane;
                    if (lane < 16 && e < p.k_k) {
                        tok_o = lists_in_lds ? ((const lds_int*)s_lk)[e] : idx_k[e];
                        info_o = lists_in_lds ? find_sorted_lds((const lds_int*)s_lv, p.k_v, tok_o) : find_sorted(idx_v, p.k_v, tok_o);
                        if (info_o < 0) load_codes(cv + (int64_t)tok_o * M, codes_o);
                    }
                } else {
                    const int j = 32 * (T - ntk) + lane;
                    if (lane < 32 && j < p.k_v) {
                        tok_o = lists_in_lds ? ((const lds_int*)s_lv)[j] : idx_v[j];
                        const int f = lists_in_lds ? find_sorted_lds((const lds_int*)s_lk, p.k_k, tok_o) : find_sorted(idx_k, p.k_k, tok_o);
                        info_o = f >= 0 ? 1 : 0;
                        if constexpr (GIVEN) pre_sc = load_score(tok_o);
                        else load_codes(ck + (int64_t)tok_o * M, codes_o);
                    }
                }
            };
            resolve_tile(T_first, pre_tok, pre_info, pre_codes);
            if constexpr (LONG) resolve_tile(T_first + p.S * kDaWaves, pre2_tok, pre2_info, pre2_codes);
            // further tiles (a wave takes more than one when the lists are long for the number of workgroups): one
            // thread per entry, the answers go through global memory
            int32_t* info_bg = p.info + (int64_t)bg * (p.k_k + p.k_v);
            const int tiles_wg = n_atiles > sp ? (n_atiles - sp + p.S - 1) / p.S : 0;
            constexpr int kOwnTiles = LONG ? 2 : 1;                  // tiles per wave that the waves resolve themselves
            if (tiles_wg > kOwnTiles * kDaWaves) {
            for (int li = tid + 64 * kOwnTiles * kDaWaves; li < 64 * tiles_wg; li += kDaThreads) {
                const int T = sp + p.S * (li >> 6), u = li & 63;
                if (T < ntk) {
                    const int e = 16 * T + u;
                    if (u < 16 && e < p.k_k) {
                        info_bg[e] = lists_in_lds ? find_sorted_lds((const lds_int*)s_lv, p.k_v, ((const lds_int*)s_lk)[e])
                                                  : find_sorted(idx_v, p.k_v, idx_k[e]);
                    }
                } else {
                    const int j = 32 * (T - ntk) + u;
                    if (u < 32 && j < p.k_v) {
                        const int f = lists_in_lds ? find_sorted_lds((const lds_int*)s_lk, p.k_k, ((const lds_int*)s_lv)[j])
                                                   : find_sorted(idx_k, p.k_k, idx_v[j]);
                        info_bg[p.k_k + j] = f >= 0 ? 1 : 0;
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the answers are in memory before the barrier that precedes their readers
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
        // LUT[m][c][h] = c1 * q_h[m*d : (m+1)*d] . cb_k[g][m][c], stored as fixed point with one scale per head
        // (quantum = max|LUT_h| / 16256): the per-token sum over sub-spaces is then exact integer arithmetic and
        // the table error is uniform instead of growing with the entry's magnitude as it would in fp16.
        // An entry is two signed bytes (lo, -hi) with value lo + 128 * hi, so that the int8 MFMA of the stream
        // loop can sum entries with the weights (1, -128).
        float val[NJ][kNH];
        float amax[kNH] = {0.f, 0.f, 0.f, 0.f};
        const bool ent_on = (DSUB != 16) || kgrp < 2;       // d = 16: only blocks 0 and 1 carry sub-spaces
#pragma unroll
        for (int j = 0; j < (GIVEN ? 0 : NJ); ++j) {
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
        for (int h = 0; h < (GIVEN ? 0 : kNH); ++h) {
            const float wm = wave_max_uniform(amax[h]);
            if (lane == 0) s_red[wave * 8 + h] = wm;
        }
        lds_barrier();
        float inv_q[kNH], quantum[kNH];
        if constexpr (!GIVEN) {
            const int hh = lane >> 4, ws = lane & 15;
            const float r_r = row16_max((ws < kDaWaves) ? s_red[ws * 8 + hh] : 0.f);
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float r = lane_bcast(r_r, 16 * h);
                if constexpr (WIDE) quantum[h] = (r > 0.f) ? r / kLutMax : 1.0f;
                // the table quantum is parked in LDS until the stream starts (keeps registers free for the anchors)
                if (tid == 0) ((float*)s_misc)[12 + h] = (r > 0.f) ? r / kLutMax : 1.0f;
                inv_q[h] = (r > 0.f) ? kLutMax / r : 0.f;
            }
        }
        uint2_t* s_lut = (uint2_t*)(smem + L::lut);
        uint2_t ent[NJ];
#pragma unroll
        for (int j = 0; j < (GIVEN ? 0 : NJ); ++j) {
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
        if (!GIVEN && ent_on) {
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
        if constexpr (WIDE) {
            // Residual entries, in units of quantum / (2 kLutMax) (|.| <= kLutMax), replace the odd copies: copy c of
            // sub-space m is then the pair of slots m + 2 M c (first entry) and m + M + 2 M c (residual).
            static_assert(!WIDE || REPS >= 2, "the residual entries live in the slots of the copies");
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                uint32_t hw[kNH];
#pragma unroll
                for (int h = 0; h < kNH; ++h) {
                    const float first = rintf(val[j][h] * inv_q[h]);
                    const int qv = (int)rintf((val[j][h] - first * quantum[h]) * (inv_q[h] * (2.f * kLutMax)));
                    const int hi = (qv + 64) >> 7;
                    const int lo = qv - 128 * hi;
                    hw[h] = ((uint32_t)lo & 0xffu) | (((uint32_t)(-hi) & 0xffu) << 8);
                }
                ent[j] = uint2_t{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16)};
            }
            if (ent_on) {
#pragma unroll
                for (int r = 0; r < NJ; ++r) {
                    const int j = (r + lane) & (NJ - 1);
                    uint2_t e = ent[0];
#pragma unroll
                    for (int jj = 1; jj < NJ; ++jj) e = (j == jj) ? ent[jj] : e;
                    const int m = (DSUB == 8) ? 4 * j + kgrp : (DSUB == 16 ? 2 * j + kgrp : 8 * (j >> 1) + 2 * kgrp + (j & 1));
#pragma unroll
                    for (int rep = 0; rep < REPS; ++rep) {
                        const int copy = (rep + (lane >> 2)) & (REPS - 1);
                        if (copy & 1) s_lut[l_code * 32 + m + M * copy] = e;
                    }
                }
            }
        }
        // the V table is not needed before the first P.V: its loads had the whole table build to land
        {
            uint4_t* dst = (uint4_t*)(smem + L::cbv);
#pragma unroll
            for (int i = 0; i < 4096 / kDaThreads; ++i) dst[tid + i * kDaThreads] = vcopy[i];
        }
        if (T_first < n_atiles) {
            if (T_first < ntk) load_k_rows(16 * T_first, pre_rows);
            else load_v_rows(32 * (T_first - ntk), pre_rows);
        }
    }
    lds_barrier();

    // m_ref: reference maximum per head (the same in every lane).  acc[a][rho]: see sm_idx below.
    float m_ref[kNH];
#pragma unroll
    for (int h = 0; h < kNH; ++h) m_ref[h] = kEmptyRef;
    float4_t acc_anchor[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};   // what the anchor entries hand to acc[a][0]
    float l_own = 0.f;                                            // sum of weights, head lane % 4, this lane's share
    // P.V of the code stream runs on the 2:4-sparse MFMA (16x16x64 f16).  Its 64 k positions form 16 groups of four;
    // the position inside a group is the class, and row 4 cls + h of the sparse operand keeps, in every group, only
    // the position of its own class: a softmax weight of head h.  All 16 rows carry useful work, and the compressed
    // operand is just four zero-extended fp16 weights per lane (the index register, a per-lane constant, says
    // where they sit).  The four positions of a group are FOUR tokens (one per class), position cls carrying slab
    // 4 a + (cls + rho) % 4 of its token; MFMA (a, rho) accumulates into acc[a][rho], whose row (cls, h) is therefore
    // slab 4 a + (cls + rho) % 4 summed over the tokens of class cls.
    // Operand geometry: compressed dword p of a lane in k-group ga pairs with the dense operand's k-group
    // 2 (ga % 2) + p / 2, elements 4 (2 (ga / 2) + p % 2) .. + 3.
    const int sm_idx = (int)(0x1111u * (uint32_t)(tj | ((tj ^ 1) << 2)));
    const uint32_t lds0 = (uint32_t)(uintptr_t)lsm;

    // ---- K side of a 64-token tile (used by the stream and by the anchor entries that have no FP16 K row).
    // Lane L handles token L of the tile; the token's class is c = L / 16 and its rank r = L % 16.  The int8 MFMA
    // leaves lane (4 c + h, k-group g) with head h's scores of tokens (c, 4 g + i), i = 0..3: from there on a lane
    // works for one head (tq) and one class (tj).
    // K gather: this lane visits sub-space (step XOR xr) mod M at every step and reads slot (step XOR xr)
    // (the constants are made where they are used, for the anchors and again for the stream: holding them across
    // the anchor entries would cost the registers those need)
    struct KConst {
        uint32_t ksel[4], kc[CW];
        int4_t k_wgt;
        uint32_t kr;
        float lut_q;
    };
    static_assert(L::lut == 0, "the table gather address is an absolute LDS address below 64 KB");
    auto make_kconst = [&](int ln) -> KConst {
        KConst c;
        const uint32_t xr = ln & 31;
        c.kr = xr & (M - 1);                                         // XOR applied to the code byte index
#pragma unroll
        for (int j = 0; j < 4; ++j) c.ksel[j] = 0x0c0c0000u | ((4u + (uint32_t)(j ^ (c.kr & 3))) << 8) | (uint32_t)j;
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            c.kc[i] = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) c.kc[i] |= ((xr ^ (uint32_t)(4 * i + j)) << 3) << (8 * j);
        }
        // constant operand of the int8 MFMA: column 4 g + h takes, from k-group g only, the (lo, hi) bytes of head h
        // with the weights (1, -128)
        const int col_blk = (ln & 15) >> 2, col_h = ln & 3, kg = ln >> 4;
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
            uint32_t wv = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = 4 * dw + j;                              // byte of the 16-byte operand
                const uint32_t wt = (i & 1) ? 0x80u : 0x01u;           // -128 on hi bytes, 1 on lo bytes
                if (kg == col_blk && ((i & 7) >> 1) == col_h) wv |= wt << (8 * j);
            }
            c.k_wgt[dw] = (int)wv;
        }
        // the table quantum of this lane's head
        c.lut_q = ((const float*)s_misc)[12];
#pragma unroll
        for (int h = 1; h < kNH; ++h) c.lut_q = (col_h == h) ? ((const float*)s_misc)[12 + h] : c.lut_q;
        return c;
    };
    // integer scores (in table quanta) of the tile whose K code dwords are kw_in, lane = token
    auto k_scores = [&](const KConst& c, const uint32_t (&kw_in)[CW], auto&& after_gathers) -> int4_t {
        // Code dwords are XOR-permuted so that step s finds the code of sub-space (s XOR kr) at a compile-time
        // register and a per-lane constant byte selector.
        if constexpr (GIVEN) {                                           // no table: the caller has the scores
            after_gathers();
            return int4_t{0, 0, 0, 0};
        }
        uint32_t kw[CW];
#pragma unroll
        for (int i = 0; i < CW; ++i) kw[i] = kw_in[i];
#pragma unroll
        for (int bit = 0; (4 << bit) < M; ++bit) {
            const bool sw = (c.kr >> (2 + bit)) & 1u;
#pragma unroll
            for (int i = 0; i < CW; ++i) {
                if (!(i & (1 << bit))) {
                    const uint32_t a = kw[i], b2 = kw[i | (1 << bit)];
                    kw[i] = sw ? b2 : a;
                    kw[i | (1 << bit)] = sw ? a : b2;
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
                ent[u] = *(const lds_uint2*)(uintptr_t)__builtin_amdgcn_perm(kw[st >> 2], c.kc[st >> 2], c.ksel[st & 3]);
            }
            __builtin_amdgcn_sched_barrier(0);                           // nothing moves across: gathers first, then the MFMAs
            if (s0 + KB >= M) after_gathers();                           // the codes are used up: the caller may reload them
#pragma unroll
            for (int u = 0; u < KB; u += 2)
                si = __builtin_amdgcn_mfma_i32_16x16x64_i8(int4_t{(int)ent[u][0], (int)ent[u][1], (int)ent[u + 1][0], (int)ent[u + 1][1]},
                                                           c.k_wgt, si, 0, 0, 0);
        }
        return si;
    };
    // Wide table: the second walk's constants (the slot's table bit flipped) and the combination of the two walks.  A lane's
    // first walk summed first entries if bit log2(M) of its own number (mod 32) is clear, residuals otherwise; after the
    // MFMA's transposition the token of register i sat in lane 16 tj + 4 kgrp + i.
    auto other_table = [&](const KConst& c) -> KConst {
        KConst c2 = c;
#pragma unroll
        for (int i = 0; i < CW; ++i) c2.kc[i] = c.kc[i] ^ (0x01010101u * (uint32_t)(M << 3));
        return c2;
    };
    auto wide_x = [&](const KConst& c, const int4_t& si, const int4_t& sj, float base, float (&x)[4]) {
        const bool swapped = (M == 16) ? (tj & 1) : (kgrp >> 1);
        const float q2 = c.lut_q * (1.0f / (2.f * kLutMax));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int first = swapped ? sj[i] : si[i], resid = swapped ? si[i] : sj[i];
            x[i] = fmaf((float)resid, q2, fmaf((float)first, c.lut_q, base));
        }
    };
    // max / sum over the lanes that work for the same head (lane % 4), result in all of them
    auto head_max = [&](float v) -> float {
        v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x124, 0xf, 0xf, true)));   // row_ror:4
        v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x128, 0xf, 0xf, true)));   // row_ror:8
        v = fmaxf(v, __shfl_xor(v, 16, 64));
        return fmaxf(v, __shfl_xor(v, 32, 64));
    };
    auto head_sum = [&](float v) -> float {
        v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x124, 0xf, 0xf, true));
        v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x128, 0xf, 0xf, true));
        v += __shfl_xor(v, 16, 64);
        return v + __shfl_xor(v, 32, 64);
    };

    // ================================================================================== anchors
    // Entries of the two anchor lists.  A K entry (token t, FP16 K row) needs V_eff(t): the FP16 V row if t is in the
    // V list too, else the centroids of t's V codes.  A V entry (token t, FP16 V row) whose token is not a K anchor
    // needs the score of t's K codes.  Tiles of entries are dealt round-robin to the workgroups (balanced by list
    // index, not by position: anchors cluster at the head and tail of a context) and statically to the waves: wave w
    // takes the workgroup's tiles w, w + 16, ... before it joins the stream.
    //   K tile (16 entries)  scores q.K_row on the dense MFMA, the K rows going straight from global memory into the
    //                        operand (entry along n, 8 channels per lane);
    //   V tile (32 entries)  scores from the K codes through the lookup table, exactly as the stream does it.
    // Values: a lane owns channels 2 lane, 2 lane + 1 of all four heads.  Per pair of entries it holds its two channels of
    // both rows (of the FP16 row: one coalesced 256-byte load per entry; of the centroids: from the V table in LDS, the
    // entry's code bytes being staged in the wave's area), and the pair's weights come back from the staging area as
    // fp16 pairs: one packed dot product per head and channel adds two entries.
    // code loads run one tile ahead of their use: HBM latency hides behind the previous tile's work
    // (addresses are a uniform base, the range's first token, plus a 32-bit offset: a range has at most 32768 tokens;
    // an empty range reads token 0)
    const int64_t n_tiles = (t1 - t0 + 63) >> 6;
    const int64_t t0c = n_tiles > 0 ? t0 : 0;
    const uint8_t* ck0 = ck + t0c * M;
    const uint8_t* cv0 = cv + t0c * M;
    const uint32_t last_rel = n_tiles > 0 ? (uint32_t)(p.N - 1 - t0) : 0u;     // tokens past the end are masked, not skipped
    float4_t sc_next = {0.f, 0.f, 0.f, 0.f};                 // given scores: head tq of tokens (tj, 4 kgrp + i) of the next tile
    const float4_t* sc0 = nullptr;
    if constexpr (GIVEN) sc0 = (const float4_t*)p.codes_k + (int64_t)bg * ((p.N + 63) & ~63LL) + t0c + (16 * tj + 4 * kgrp + tq);
    auto load_tile = [&](int tile, uint32_t (&kw_)[CW], uint32_t (&vw_)[CW]) {
        uint32_t rel = (uint32_t)tile * 64u + (uint32_t)lane;
        rel = rel < last_rel ? rel : last_rel;
        const uint32_t off = rel * (uint32_t)M;
        if constexpr (GIVEN) {
            sc_next = sc0[(uint32_t)tile * 64u];
            load_codes(cv0 + off, vw_);
        } else if (CW == 2) {
            const uint2_t a = *(const uint2_t*)(ck0 + off), c = *(const uint2_t*)(cv0 + off);
            kw_[0] = a[0]; kw_[1] = a[1]; vw_[0] = c[0]; vw_[1] = c[1];
        } else {
#pragma unroll
            for (int i = 0; i < CW / 4; ++i) {
                const uint4_t a = *(const uint4_t*)(ck0 + off + 16 * i), c = *(const uint4_t*)(cv0 + off + 16 * i);
#pragma unroll
                for (int e = 0; e < 4; ++e) { kw_[4 * i + e] = a[e]; vw_[4 * i + e] = c[e]; }
            }
        }
    };
    uint32_t kw_next[CW], vw_next[CW];
    if (T_first < n_atiles) {
        typedef __attribute__((address_space(3))) uint8_t lds_u8;
        typedef __attribute__((address_space(3))) uint32_t lds_u32;
        typedef __attribute__((address_space(3))) uint2_t lds_u32x2;
        typedef __attribute__((address_space(3))) uint4_t lds_u32x4;
        const int32_t* info_bg = p.info + (int64_t)bg * (p.k_k + p.k_v);
        const half_t* s_qh = (const half_t*)(smem + L::qh);               // Q as MFMA A operand: row = head
        float l_lane[kNH] = {0.f, 0.f, 0.f, 0.f};                        // K tiles: per-lane shares of the weight sums, per head
        float av[kNH][2];                                                // value sums: head h, channels 2 lane, 2 lane + 1
#pragma unroll
        for (int h = 0; h < kNH; ++h) av[h][0] = av[h][1] = 0.f;
        const uint32_t stg_b = lds0 + (uint32_t)(L::pst + wave * kStgBytes);      // staged code rows: [entry][M] bytes
        static_assert(32 * M <= kStgBytes, "the code rows of a K tile fit the wave's staging area");
        const uint32_t m_lane = (uint32_t)(2 * lane) / DSUB;                      // sub-space of this lane's two channels
        const uint32_t vtab = lds0 + (uint32_t)L::cbv + 4u * (uint32_t)lane;      // + code << 8: this lane's channels of a centroid row
        // weights of a tile's entries, for the value sums: fp16 pairs of two consecutive entries, [pair][head] (16 bytes per
        // pair, read back by all lanes at once); after the code rows in the staging area
        constexpr int kWOff = 1024;
        static_assert(32 * M <= kWOff && kWOff + 32 * 16 <= kStgBytes, "code rows and weights share the wave's staging area");
        const uint32_t stg_wt = stg_b + kWOff;
        // adds entries t, t + 1 (weights of pair `pair`, this lane's two channels of their V rows in va, vb)
        auto add_pair = [&](int pair, uint32_t va_, uint32_t vb_) {
            const uint4_t w4 = *(const lds_u32x4*)(uintptr_t)(stg_wt + 16u * (uint32_t)pair);
            const half2_t lo = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(vb_, va_, 0x05040100u));   // channel 2 lane of both entries
            const half2_t hi = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(vb_, va_, 0x07060302u));   // channel 2 lane + 1
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const uint32_t w_h = w4[h];   // (a bit_cast taken straight from the vector element reads element 0 for every h)
                const half2_t wh = __builtin_bit_cast(half2_t, w_h);
                av[h][0] = __builtin_amdgcn_fdot2(lo, wh, av[h][0], false);
                av[h][1] = __builtin_amdgcn_fdot2(hi, wh, av[h][1], false);
            }
        };
        auto pack2 = [](float a, float b) -> uint32_t {
            return (uint32_t)__builtin_bit_cast(unsigned short, (half_t)a) | ((uint32_t)__builtin_bit_cast(unsigned short, (half_t)b) << 16);
        };
        // moves the reference maxima to cover a tile whose largest scores are m_tile[h], rescaling what was summed so far
        auto move_reference = [&](const float (&m_tile)[kNH]) {
            float a_own = 1.f;
#pragma unroll
            for (int h = 0; h < kNH; ++h) {
                const float m_new = fmaxf(m_ref[h], m_tile[h] - kPShift);
                const float alpha = fast_exp2(m_ref[h] - m_new);
                l_lane[h] *= alpha;
                av[h][0] *= alpha;
                av[h][1] *= alpha;
                a_own = (tq == h) ? alpha : a_own;
                m_ref[h] = m_new;
            }
            l_own *= a_own;
        };
        for (int T = T_first; T < n_atiles; T += p.S * kDaWaves) {
            // the tile's tokens, cross membership, code rows and FP16 rows are in pre_tok, pre_info, pre_codes, pre_rows
            // (the first tile's since the prologue, a further tile's since the end of the tile before)
            if (T < ntk) {
                // ------------------------------------------------------------------ K tile: entries 32 T .. 32 T + 31
                const int e0 = 16 * T;
                int my_tok = 0, my_part = -1, my_valid = 0;               // lanes 0..15 each own one entry
                if (lane < 16 && e0 + lane < p.k_k) { my_valid = 1; my_tok = pre_tok; my_part = pre_info; }
                uint4_t kb[4];
#pragma unroll
                for (int st = 0; st < 4; ++st) kb[st] = uint4_t{pre_rows[4 * st], pre_rows[4 * st + 1], pre_rows[4 * st + 2], pre_rows[4 * st + 3]};
                // V code rows of the entries without an FP16 V row
                __builtin_amdgcn_wave_barrier();                           // the previous tile's readers are done
                if (my_valid && my_part < 0) {
                    if constexpr (CW == 2) {
                        *(lds_u32x2*)(uintptr_t)(stg_b + 8u * lane) = uint2_t{pre_codes[0], pre_codes[1]};
                    } else {
#pragma unroll
                        for (int i = 0; i < CW / 4; ++i)
                            *(lds_u32x4*)(uintptr_t)(stg_b + (uint32_t)(4 * CW) * lane + 16u * i) =
                                uint4_t{pre_codes[4 * i], pre_codes[4 * i + 1], pre_codes[4 * i + 2], pre_codes[4 * i + 3]};
                    }
                }
                // scores: lanes 0..15 hold head r of entry lane
                float sc[4];
                {
                    float4_t c4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int st = 0; st < 4; ++st) {
                        half8_t qa = *(const half8_t*)(s_qh + (arow & 3) * kD + 32 * st + 8 * kgrp);
                        if (arow >= kNH) qa = half8_t{0, 0, 0, 0, 0, 0, 0, 0};
                        c4 = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa, __builtin_bit_cast(half8_t, kb[st]), c4, 0, 0, 0);
                    }
                    const bool on = kgrp == 0 && e0 + arow < p.k_k;
#pragma unroll
                    for (int r = 0; r < 4; ++r) sc[r] = on ? c4[r] * p.c1 : kNegBig;
                }
                float m_tile[kNH];
#pragma unroll
                for (int h = 0; h < kNH; ++h) m_tile[h] = wave_max_uniform(sc[h]);
                move_reference(m_tile);
                float pw[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pw[r] = fast_exp2(sc[r] - m_ref[r]);                  // 0 for lanes without an entry
                    l_lane[r] += pw[r];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();                           // the staged code rows are visible
                // values.  The weights go to the staging area as fp16 pairs (lane n holds entry n: even lanes pair up
                // with their right neighbour).  First pass, all 16 entries without a branch: the centroids of the staged
                // codes, with weight zero where the entry has an FP16 V row (or does not exist).  Second pass, only if there
                // is such an entry: the FP16 rows, with the weights of exactly those entries.
                const unsigned long long both64 = __ballot(my_part >= 0);
                auto put_weights = [&](bool coded_pass) {
                    const bool mine = (((both64 >> arow) & 1ull) == 0ull) == coded_pass;
                    uint4_t w4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float a = mine ? pw[r] : 0.f;
                        const float b = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, a), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
                        w4[r] = pack2(a, b);
                    }
                    if (kgrp == 0 && (lane & 1) == 0) *(lds_u32x4*)(uintptr_t)(stg_wt + 16u * (uint32_t)(arow >> 1)) = w4;
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                };
                put_weights(true);
#pragma unroll
                for (int tb = 0; tb < 16; tb += 8) {
                    uint32_t code[8], v2[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) code[k] = *(const lds_u8*)(uintptr_t)(stg_b + (uint32_t)((tb + k) * M) + m_lane);
#pragma unroll
                    for (int k = 0; k < 8; ++k) v2[k] = *(const lds_u32*)(uintptr_t)(vtab + (code[k] << 8));
#pragma unroll
                    for (int k = 0; k < 8; k += 2) add_pair((tb + k) >> 1, v2[k], v2[k + 1]);
                }
                if (both64 != 0ull) {
                    __builtin_amdgcn_wave_barrier();
                    put_weights(false);
#pragma unroll 1
                    for (int pr = 0; pr < 8; ++pr) {
                        if (((both64 >> (2 * pr)) & 3ull) == 0ull) continue;
                        uint32_t v2[2];
#pragma unroll
                        for (int k = 0; k < 2; ++k) {
                            const int part = __builtin_amdgcn_readlane(my_part, 2 * pr + k);
                            v2[k] = 0u;
                            if (part >= 0) v2[k] = *(const uint32_t*)(p.rows_v + ((int64_t)bg * p.k_v + part) * kD + 2 * lane);
                        }
                        add_pair(pr, v2[0], v2[1]);
                    }
                }
            } else {
                // ------------------------------------------------------------------ V tile: entries 64 (T - ntk) + lane
                const int j0 = 32 * (T - ntk);
                const bool in_list = lane < 32 && j0 + lane < p.k_v;
                int tok = 0, skip = 1;
                if (in_list) { tok = pre_tok; skip = pre_info; }
                (void)tok;
                const uint32_t (&va)[32] = pre_rows;
                const uint32_t (&kw)[CW] = pre_codes;
                const unsigned long long keep64 = __ballot(skip == 0);     // entries to process
                int ln = lane;
                asm volatile("" : "+v"(ln));                               // (a value of its own: not merged with the stream's copy)
                const KConst kcst = make_kconst(ln);
                const int4_t si = k_scores(kcst, kw, [] {});
                // register i of lane (4 c + h, g) = entry 16 c + 4 g + i, head h (classes 2 and 3 are empty: keep bits 0)
                const uint32_t keep_bits = (uint32_t)(keep64 >> (32 * (tj >> 1) + 16 * (tj & 1) + 4 * kgrp));
                float sr[4], lm = kNegBig;
                if constexpr (WIDE) {
                    const int4_t sj = k_scores(other_table(kcst), kw, [] {});
                    wide_x(kcst, si, sj, 0.f, sr);
                }
                if constexpr (GIVEN) {
                    // lane = entry holds its token's four scores: through the staging area into the form above
                    __builtin_amdgcn_wave_barrier();
                    if (lane < 32) *(lds_u32x4*)(uintptr_t)(stg_b + 16u * (uint32_t)lane) = __builtin_bit_cast(uint4_t, pre_sc);
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        sr[i] = 0.f;
                        if (tj < 2) sr[i] = __builtin_bit_cast(float, *(const lds_u32*)(uintptr_t)(stg_b + 16u * (uint32_t)(16 * tj + 4 * kgrp + i) + 4u * (uint32_t)tq));
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (!WIDE && !GIVEN) sr[i] = (float)si[i] * kcst.lut_q;
                    lm = fmaxf(lm, ((keep_bits >> i) & 1u) ? sr[i] : kNegBig);
                }
                lm = head_max(lm);
                float m_tile[kNH];
#pragma unroll
                for (int h = 0; h < kNH; ++h) m_tile[h] = lane_bcast(lm, h);       // lanes 0..3 work for heads 0..3
                move_reference(m_tile);
                float neg_m = -m_ref[0];
#pragma unroll
                for (int h = 1; h < kNH; ++h) neg_m = (tq == h) ? -m_ref[h] : neg_m;
                float pw[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pw[i] = ((keep_bits >> i) & 1u) ? fast_exp2(sr[i] + neg_m) : 0.f;
                    l_own += pw[i];
                }
                // values: register i of lane (4 c + h, g) is entry 16 c + 4 g + i, so a lane holds two pairs of its head
                __builtin_amdgcn_wave_barrier();
                *(lds_u32*)(uintptr_t)(stg_wt + 16u * (uint32_t)(8 * tj + 2 * kgrp) + 4u * (uint32_t)tq) = pack2(pw[0], pw[1]);
                *(lds_u32*)(uintptr_t)(stg_wt + 16u * (uint32_t)(8 * tj + 2 * kgrp + 1) + 4u * (uint32_t)tq) = pack2(pw[2], pw[3]);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int k = 0; k < 32; k += 2) add_pair(k >> 1, va[k], va[k + 1]);
            }
            // a further tile of this wave: fetch it the plain way (its cross membership was worked out in the prologue)
            const int Tn = T + p.S * kDaWaves;
            if (LONG && Tn < n_atiles && T == T_first) {
                // the second tile: tokens, cross membership and code rows are there since the prologue
                pre_tok = pre2_tok;
                pre_info = pre2_info;
#pragma unroll
                for (int i = 0; i < CW; ++i) pre_codes[i] = pre2_codes[i];
                if (Tn < ntk) load_k_rows(16 * Tn, pre_rows);
                else load_v_rows(32 * (Tn - ntk), pre_rows);
            } else if (Tn < n_atiles) {
#pragma unroll
                for (int i = 0; i < CW; ++i) pre_codes[i] = 0u;
                if (Tn < ntk) {
                    const int e = 16 * Tn + lane;
                    if (lane < 16 && e < p.k_k) {
                        pre_tok = idx_k[e];
                        pre_info = info_bg[e];
                        if (pre_info < 0) load_codes(cv + (int64_t)pre_tok * M, pre_codes);
                    }
                    load_k_rows(16 * Tn, pre_rows);
                } else {
                    const int j = 32 * (Tn - ntk) + lane;
                    if (lane < 32 && j < p.k_v) {
                        pre_tok = idx_v[j];
                        pre_info = info_bg[p.k_k + j];
                        if constexpr (GIVEN) pre_sc = load_score(pre_tok);
                        else load_codes(ck + (int64_t)pre_tok * M, pre_codes);
                    }
                    load_v_rows(32 * (Tn - ntk), pre_rows);
                }
            }
        }
        // hand over to the stream's forms.  Weight sums: head lane % 4 in each lane (the K tiles' share goes to lanes 0..3).
#pragma unroll
        for (int h = 0; h < kNH; ++h) {
            const float t = wave_sum(l_lane[h]);
            l_own += (lane == h) ? t : 0.f;
        }
        // Value sums: into the accumulators of MFMA (a, 0), whose register h in lane (n, cls) is head h, channel
        // 16 (4 a + cls) + n.  Two heads at a time through the wave's staging area.
        float* s_f = (float*)(smem + L::pst + wave * kStgBytes);            // [2][128] fp32
        static_assert(2 * kD * 4 <= kStgBytes, "two heads of value sums fit the wave's staging area");
#pragma unroll
        for (int hp = 0; hp < 2; ++hp) {
            __builtin_amdgcn_wave_barrier();
            *(float2*)(s_f + 2 * lane) = float2{av[2 * hp][0], av[2 * hp][1]};
            *(float2*)(s_f + kD + 2 * lane) = float2{av[2 * hp + 1][0], av[2 * hp + 1][1]};
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                acc_anchor[a][2 * hp] = s_f[16 * (4 * a + kgrp) + (lane & 15)];
                acc_anchor[a][2 * hp + 1] = s_f[kD + 16 * (4 * a + kgrp) + (lane & 15)];
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    // ================================================================================== stream
    float4_t acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int rho = 0; rho < 4; ++rho) acc[a][rho] = rho == 0 ? acc_anchor[a] : float4_t{0.f, 0.f, 0.f, 0.f};
    {
        const KConst kcst = make_kconst(lane);
        // V gather address = table base | code << 8 | byte offset of the 8-byte piece inside the code's row, the piece
        // being chunk tq of slab 4 a + (tj + rho) % 4 (128 a goes into the instruction's immediate): one byte permute
        // of a staged code dword and a per-lane constant
        static_assert((L::cbv & 0xffff) == 0, "the V table base must be a multiple of 64 KB");
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

        // this lane's head: running reference
        float neg_m = -m_ref[0];
#pragma unroll
        for (int h = 1; h < kNH; ++h) neg_m = (tq == h) ? -m_ref[h] : neg_m;

        // One tile.  Its codes are in kw_in / vw; once they are used up (K codes by the table gathers, V codes by the
        // staging write; d = 4 stages its second half in the V phase) `reload` puts the next tile's codes into the same
        // registers, so that nothing is copied between tiles.
        auto do_tile = [&](int tile, uint32_t (&kw_in)[CW], uint32_t (&vw)[CW], auto&& reload) {
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

            // ---- K side: scores in table quanta
            // (wide table: two walks; the codes may be reloaded once the second walk's gathers are issued)
            float sg[4] = {0.f, 0.f, 0.f, 0.f};                       // given scores: taken before the reload replaces them
            if constexpr (GIVEN) {
#pragma unroll
                for (int i = 0; i < 4; ++i) sg[i] = sc_next[i];
            }
            const int4_t si = k_scores(kcst, kw_in, [&] { if constexpr (DSUB != 4 && !WIDE) reload(); });
            int4_t sj = {0, 0, 0, 0};
            if constexpr (WIDE) sj = k_scores(other_table(kcst), kw_in, [&] { reload(); });
            // ---- softmax: register i = token (tj, 4 kgrp + i), head tq.  x = score - reference.
            const uint32_t keep_bits = ~mw >> mask_sh;                 // bit i set: token i is neither anchored nor past the range
            float x[4];
            if constexpr (GIVEN) {
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = sg[i] + neg_m;
            } else if constexpr (WIDE) {
                wide_x(kcst, si, sj, neg_m, x);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = fmaf((float)si[i], kcst.lut_q, neg_m);
            }
            if (__any(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])) > kPShift)) {
                // some score exceeds the running maximum by more than the head room: move the reference, rescale
                float lm = kNegBig;
#pragma unroll
                for (int i = 0; i < 4; ++i) lm = fmaxf(lm, ((keep_bits >> i) & 1u) ? x[i] : kNegBig);
                lm = head_max(lm);                                      // largest unmasked x of head tq in the tile
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
                if constexpr (GIVEN) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = sg[i] + neg_m;
                } else if constexpr (WIDE) {
                    wide_x(kcst, si, sj, neg_m, x);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = fmaf((float)si[i], kcst.lut_q, neg_m);
                }
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
            // 4 a + (tj + rho) % 4, the four rows of a transposed read being the four classes.  The operand reads of
            // kVDepth MFMAs are in flight at any time: a wave has few neighbours on its SIMD to hide the LDS latency.
            if constexpr (DSUB != 4) {
                uint32_t vt[2][4][2];                                  // staged code dwords: [half][element quad][dword]
#pragma unroll
                for (int a = 0; a < (DSUB == 8 ? 2 : 1); ++a)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const uint32_t ad = ((e4 >> 1) ? stg_r1 : stg_r0) + (uint32_t)(SU * (e4 & 1)) + 8u * a;
                        const uint2_t r = *(const lds_uint2*)(uintptr_t)ad;
                        vt[a][e4][0] = r[0]; vt[a][e4][1] = r[1];
                    }
                auto fetch = [&](int u, half4_t (&vb)[4]) {
                    const int a = u >> 2, rho = u & 3;
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        uint32_t ad;
                        if constexpr (DSUB == 8) ad = __builtin_amdgcn_perm(vt[a][e4][rho >> 1], v_const[rho], v_sel[rho & 1]);
                        else ad = __builtin_amdgcn_perm(vt[0][e4][a], v_const[rho], 0x0c020000u | ((4u + (uint32_t)rho) << 8));
                        vb[e4] = lds_read_tr16_abs(ad + 128 * a);
                    }
                };
                constexpr int kVDepth = 3;
                half4_t vb[kVDepth][4];
#pragma unroll
                for (int u = 0; u < kVDepth; ++u) fetch(u, vb[u]);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    half4_t (&cur)[4] = vb[u % kVDepth];
                    const half16_t bop = {cur[0][0], cur[0][1], cur[0][2], cur[0][3], cur[1][0], cur[1][1], cur[1][2], cur[1][3],
                                          cur[2][0], cur[2][1], cur[2][2], cur[2][3], cur[3][0], cur[3][1], cur[3][2], cur[3][3]};
                    acc[u >> 2][u & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(pa, bop, acc[u >> 2][u & 3], sm_idx, 0, 0);
                    if (u + kVDepth < 8) fetch(u + kVDepth, vb[u % kVDepth]);
                }
            } else {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    uint32_t vt[4][4];
                    if (a == 1) {
                        __builtin_amdgcn_wave_barrier();
                        stage_d4(1);
                        reload();
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4) {
                        const uint32_t ad = ((e4 >> 1) ? stg_r1 : stg_r0) + (uint32_t)(SU * (e4 & 1));
                        const uint4_t r = *(const __attribute__((address_space(3))) uint4_t*)(uintptr_t)ad;
#pragma unroll
                        for (int u = 0; u < 4; ++u) vt[e4][u] = r[u];
                    }
                    auto fetch = [&](int rho, half4_t (&vb)[4]) {
#pragma unroll
                        for (int e4 = 0; e4 < 4; ++e4)
                            vb[e4] = lds_read_tr16_abs(__builtin_amdgcn_perm(vt[e4][rho], v_const[rho], v_sel[0]) + 128 * a);
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
            }
            __builtin_amdgcn_wave_barrier();
        };

        // The next tile's codes are requested while the current tile is worked on (from the middle of its K phase).  The
        // request is unconditional: a wave that has no further tile re-reads the range's last one.  The next tile's number
        // comes from the workgroup's counter; the fetch-add is issued at the top of a tile and read where the request is
        // made, so that its LDS round trip is off the critical path.
        int tile = wave;                                              // the first tile of wave w is tile w
        const int nt = (int)n_tiles;
        const uint32_t tile_ctr = lds0 + (uint32_t)(L::red + kDaWaves * 32 + 8 * 4);      // LDS address of s_misc[8]
        load_tile(tile < nt ? tile : nt - 1, kw_next, vw_next);
        while (tile < nt) {
            // (the fetch-add and the wait for it are written out: an atomic of the language is waited for on the spot)
            int t_raw = 0;
            if constexpr (!DET) {
                if (lane == 0) asm volatile("ds_add_rtn_u32 %0, %1, %2" : "=v"(t_raw) : "v"(tile_ctr), "v"(1) : "memory");
            }
            int tile_next = 0;
            do_tile(tile, kw_next, vw_next, [&] {
                if constexpr (DET) {
                    tile_next = tile + kDaWaves;
                } else {
                    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(t_raw) : : "memory");
                    tile_next = __builtin_amdgcn_readfirstlane(t_raw);
                }
                load_tile(tile_next < nt ? tile_next : nt - 1, kw_next, vw_next);
            });
            tile = tile_next;
        }
#pragma unroll
        for (int h = 0; h < kNH; ++h) m_ref[h] = -lane_bcast(neg_m, h);
    }
    // weight sums per head: add up the lanes that worked for the head
    float l_sum[kNH];
    {
        const float v = head_sum(l_own);
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
    size_t off_part, off_done, off_info, off_stat, total;
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
    size_t off = 0;
    pl.off_part = off; off += align_up((size_t)g.B * g.Hq * pl.S * (kD + 2) * sizeof(float));
    pl.off_done = off; off += align_up((size_t)g.B * g.Hkv * sizeof(unsigned long long));
    pl.off_info = off; off += align_up((size_t)g.B * g.Hkv * (size_t)(k_k + k_v) * sizeof(int32_t));
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

// process-wide option mask of antkv_set_decode_options (see the MODE parameter of decode_attn_kernel)
static std::atomic<int> g_options{0};

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
    p.part = part; p.out = a.out; p.done = (unsigned long long*)(w + pl.off_done); p.info = (int32_t*)(w + pl.off_info); p.tag = next_launch_tag(); p.N = a.N; p.N_cap = a.N_cap; p.k_k = (int)a.k_k; p.k_v = (int)a.k_v;
    p.c1 = a.scale * kLog2e; p.Hq = g.Hq; p.Hkv = g.Hkv; p.G = g.G; p.S = pl.S; p.chunk = pl.chunk;
    if (a.given_scores) {
        if (a.k_k != 0 || want_ans) return hipErrorInvalidValue;      // the scores cover the K anchors already
        p.codes_k = (const uint8_t*)a.given_scores;
    }
    if (pl.S > 1024) return hipErrorInvalidValue;        // the in-kernel merge keeps one weight per slot in LDS
    const size_t shmem = Lds<DSUB>::total;
    // One-time set-up per instantiation (and per process): raise the dynamic LDS limit, and make sure the kernel has
    // no static LDS — its table gathers use absolute LDS addresses, which assumes the dynamic block starts at 0.
    static const hipError_t setup = [] {
        for (const void* f : {(const void*)decode_attn_kernel<DSUB, 0>, (const void*)decode_attn_kernel<DSUB, 1>,
                              (const void*)decode_attn_kernel<DSUB, 2>, (const void*)decode_attn_kernel<DSUB, 3>,
                              (const void*)decode_attn_kernel<DSUB, 4>, (const void*)decode_attn_kernel<DSUB, 5>,
                              (const void*)decode_attn_kernel<DSUB, 6>, (const void*)decode_attn_kernel<DSUB, 7>,
                              (const void*)decode_attn_kernel<DSUB, 8>, (const void*)decode_attn_kernel<DSUB, 9>}) {
            hipFuncAttributes attr;
            hipError_t r = hipFuncGetAttributes(&attr, f);
            if (r != hipSuccess) return r;
            if (attr.sharedSizeBytes != 0) return hipErrorInvalidConfiguration;
            r = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Lds<DSUB>::total);
            if (r != hipSuccess) return r;
        }
        return hipSuccess;
    }();
    hipError_t e = setup;
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)((int64_t)g.B * g.Hkv * pl.S);
    // anchor lists between 3073 and 16384 entries go through the kernels that hold them in the table areas
    const int64_t k_max = a.k_k > a.k_v ? a.k_k : a.k_v;
    int mode = (g_options.load(std::memory_order_relaxed) & 3) | ((k_max > 3 * kDaThreads && k_max <= 16384) ? 4 : 0);   // (3 rounds of 1024 fit the staging areas)
    if (a.given_scores) mode = 8 | (mode & 1);
    switch (mode) {
    case 0: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 0>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 1: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 1>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 2: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 2>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 3: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 3>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 4: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 4>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 5: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 5>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 6: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 6>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 8: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 8>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    case 9: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 9>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    default: hipLaunchKernelGGL((decode_attn_kernel<DSUB, 7>), dim3(grid), dim3(kDaThreads), shmem, st, p); break;
    }
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

int set_decode_options(int options) { return g_options.exchange(options & 3); }

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
