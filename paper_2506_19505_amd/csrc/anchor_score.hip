// Anchor Score (paper Eq. (4); two-phase procedure of Alg. 1, Sec. 3.3):
//   AnS(V_j) = sum_i A_ij,   AnS(K_j) = sum_i A_ij (1 - A_ij) ||Q_i||_2,   A = causal softmax(scale Q K^T),
// summed over the query heads of a KV head.  A is never materialised.
//
//   phase 1  row statistics: per (head, query row) the running max and sum of exp over the visible keys.
//            MFMA tile with keys on the row axis and queries on the column axis, so a lane owns one query
//            and reduces over keys in its own registers.  Long contexts with few query rows are split
//            over the key axis; a small kernel merges the splits and adds ||Q_i||_2.
//            (Skipped when the caller supplies row max / row sum, as an extended attention kernel would.)
//   phase 2  column reduction: per (KV head, block of keys) loop over the group's heads and all query
//            tiles that can see the block, rebuild A = exp2(S*c1 - c_i) from the row statistic
//            c_i = max_i*log2(e) + log2(sum_i), and reduce over queries.  Queries sit on the MFMA row
//            axis and keys on the column axis, so a lane owns one key; per-tile partial sums are fp32,
//            the running column sums are fp64.
// All contractions are v_mfma_f32_32x32x16_f16 on the raw fp16 Q and K (exact products, fp32 accumulate);
// the softmax scale is applied to the fp32 result.
#include "common.h"

#include <type_traits>

namespace antkv {

namespace {

constexpr int kAsThreads = 512;   // 8 waves

// MFMA operand for 32 rows x 128 channels: lane (r = lane%32, kh = lane/32) holds, for each of the
// 8 k-steps s, the 8 channels 16*s + 8*kh .. +7 of row r.
struct Tile128 {
    half8_t v[8];
};

__device__ __forceinline__ void load_tile(Tile128& t, const half_t* row_ptr, int kh)
{
#pragma unroll
    for (int s = 0; s < 8; ++s) t.v[s] = *(const half8_t*)(row_ptr + 16 * s + 8 * kh);
#pragma unroll
    for (int s = 0; s < 8; ++s) pin(t.v[s]);
}

// A 32-row x 128-channel tile shared by the waves of a workgroup sits in LDS with rows padded to 136 halfs
// (272 bytes): the 16 lanes that one 16-byte LDS read serves per clock then fall on 16 different bank quads.
constexpr int kRowPad = 136;
constexpr int kTileHalfs = 32 * kRowPad;

// rows x staged tile: the staged tile is the A operand (rows of the result), the register tile the B operand
__device__ __forceinline__ float16_t tile_dot_lds_a(const half_t* __restrict__ st, const Tile128& b, int n, int kh)
{
    float16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const half8_t a = *(const half8_t*)(st + n * kRowPad + 16 * s + 8 * kh);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b.v[s], acc, 0, 0, 0);
    }
    return acc;
}

__device__ __forceinline__ float16_t tile_dot(const Tile128& a, const Tile128& b)
{
    float16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.v[s], b.v[s], acc, 0, 0, 0);
    return acc;
}

// -------------------------------------------------------------------------------------------------
// phase 1: partial row statistics.  grid = (key splits, query blocks, B*Hkv); 8 waves = HG heads of the
// group x 8/HG query tiles of 32 with HG = min(G, 4), so that no wave idles for small groups (larger groups loop).
// part: [B][Hq][Nq][KS][2] = (max in log2 units, sum of exp2)
// -------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAsThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void ans_row_stats(
    const half_t* __restrict__ q, const half_t* __restrict__ k, int64_t N, int64_t Nq, float c1,
    float* __restrict__ part, int Hq, int Hkv, int G, int KS, int64_t keys_per_split)
{
    __shared__ __attribute__((aligned(16))) half_t s_k[2][kTileHalfs];   // key tiles, double-buffered
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, kh = lane >> 5;
    const int ks = blockIdx.x;
    const int64_t qblk = blockIdx.y;
    const int b = blockIdx.z / Hkv, g = blockIdx.z % Hkv;
    const int HG = G >= 4 ? 4 : G;                              // head slots of the workgroup
    const int qspan = 32 * (8 / HG);                            // query rows per workgroup
    const int64_t q0 = qblk * qspan + (wave >> (HG >> 1)) * 32;        // first query row of this wave's tile
    const bool wave_on = q0 < Nq;
    const int64_t qi = q0 + n;                                  // this lane's query row
    const int64_t qrow = qi < Nq ? qi : Nq - 1;
    const int64_t qpos = N - Nq + qrow;                         // absolute position = last visible key
    const int64_t tile_last_pos = N - Nq + ((q0 + 31 < Nq) ? q0 + 31 : Nq - 1);
    const int64_t k_lo = (int64_t)ks * keys_per_split;
    // keys this workgroup walks: up to the last key any of its queries can see
    const int64_t blk_last_pos = N - Nq + ((qblk * qspan + qspan - 1 < Nq) ? qblk * qspan + qspan - 1 : Nq - 1);
    int64_t k_end = k_lo + keys_per_split;
    if (k_end > blk_last_pos + 1) k_end = blk_last_pos + 1;
    int64_t k_hi = k_lo + keys_per_split;                       // this wave's own limit
    if (k_hi > tile_last_pos + 1) k_hi = tile_last_pos + 1;
    const half_t* kbase = k + ((int64_t)b * Hkv + g) * N * kD;
    // staging: thread t moves 16 bytes: row t / 16, chunk t % 16 of the tile
    const int srow = tid >> 4, schunk = tid & 15;
    auto fetch = [&](int64_t kt) -> uint4_t {
        const int64_t krow = (kt + srow < N) ? kt + srow : N - 1;
        return *(const uint4_t*)(kbase + krow * kD + 8 * schunk);
    };

    for (int h_it = 0; h_it < (G + HG - 1) / HG; ++h_it) {
        const int hh = HG * h_it + (wave & (HG - 1));
        const bool head_on = wave_on && hh < G;
        const int h = g * G + (hh < G ? hh : G - 1);
        Tile128 tq;
        load_tile(tq, q + (((int64_t)b * Hq + h) * Nq + qrow) * kD, kh);
        wait_all_loads();
        float m_run = kNegBig, l_run = 0.f;
        // One-step software pipeline: the scores of tile t+1 are computed while the statistics of tile t are
        // updated, so LDS holds tiles t+1 (read) and t+2 (being written); tile t's buffer is the one rewritten.
        if (k_lo < k_end) *(uint4_t*)(&s_k[0][srow * kRowPad + 8 * schunk]) = fetch(k_lo);
        if (k_lo + 32 < k_end) *(uint4_t*)(&s_k[1][srow * kRowPad + 8 * schunk]) = fetch(k_lo + 32);
        __syncthreads();
        float16_t acc_cur;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_cur[r] = 0.f;
        if (head_on && k_lo < k_hi) acc_cur = tile_dot_lds_a(s_k[0], tq, n, kh);   // rows = keys, cols = queries
        int buf = 0;                                                // buffer of tile t
        for (int64_t kt = k_lo; kt < k_end; kt += 32) {
            const bool more = kt + 64 < k_end;
            uint4_t nxt = {0u, 0u, 0u, 0u};
            if (more) nxt = fetch(kt + 64);
            if (head_on && kt < k_hi) {
                // Exponents are taken against this lane's reference m_run, which only moves when a tile brings
                // a score more than 64 (log2 units) above it, or when the lane has seen nothing yet: the common
                // tile costs one fma, one exp2, one add and one max per element.
                const bool init = m_run > kNegBig;
                const float base = init ? m_run : 0.f;
                float arg[16];
                float mx = kNegBig, sum = 0.f;
                float16_t acc_next;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_next[r] = 0.f;
                const int lim_q = (int)(qpos - kt), lim_k = (int)(k_hi - kt);   // visible: offset <= lim_q, < lim_k
                auto body = [&](auto masked) {
                    const half_t* ap = &s_k[buf ^ 1][n * kRowPad + 8 * kh];
                    half8_t a_op[8];
                    a_op[0] = *(const half8_t*)(ap);
                    a_op[1] = *(const half8_t*)(ap + 16);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        if (s + 2 < 8) a_op[s + 2] = *(const half8_t*)(ap + 16 * (s + 2));
                        acc_next = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_op[s], tq.v[s], acc_next, 0, 0, 0);
#pragma unroll
                        for (int e2 = 0; e2 < 2; ++e2) {
                            const int r = 2 * s + e2;
                            float x = fmaf(acc_cur[r], c1, -base);
                            if (decltype(masked)::value) {
                                const int off = 8 * (r >> 2) + 4 * kh + (r & 3);
                                if (!((off <= lim_q) && (off < lim_k))) x = kNegBig;
                            }
                            arg[r] = x;
                            mx = fmaxf(mx, x);
                            sum += fast_exp2(x);
                        }
                    }
                };
                // every key of the tile is visible to every query of the wave: no mask
                if (kt + 31 <= N - Nq + q0 && kt + 31 < k_hi) body(std::false_type{});
                else body(std::true_type{});
                if (init && mx <= 64.f) {
                    l_run += sum;
                } else if (mx > 0.5f * kNegBig) {                  // the tile has a visible element: move the reference
                    float sum2 = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sum2 += fast_exp2(arg[r] - mx);
                    l_run = (init ? l_run * fast_exp2(-mx) : 0.f) + sum2;
                    m_run = base + mx;
                }
                acc_cur = acc_next;
            }
            if (more) *(uint4_t*)(&s_k[buf][srow * kRowPad + 8 * schunk]) = nxt;
            __syncthreads();
            buf ^= 1;
        }
        // merge the two half-waves (they saw complementary keys of the same query)
        const float m_o = __shfl_xor(m_run, 32, 64), l_o = __shfl_xor(l_run, 32, 64);
        const float m_f = fmaxf(m_run, m_o);
        const float l_f = l_run * fast_exp2(m_run - m_f) + l_o * fast_exp2(m_o - m_f);
        if (head_on && kh == 0 && qi < Nq) {
            float* p = part + ((((int64_t)b * Hq + h) * Nq + qi) * KS + ks) * 2;
            p[0] = m_f;
            p[1] = l_f;
        }
        __syncthreads();
    }
}

// merge key splits -> c_i = m + log2(l); also ||Q_i||_2.  One 16-lane group per (b, h, i).
__global__ __launch_bounds__(256) void ans_finalize_stats(
    const half_t* __restrict__ q, const float* __restrict__ part, int KS, const float* __restrict__ row_max,
    const float* __restrict__ row_sum, float* __restrict__ c_out, float* __restrict__ nq_out, int64_t n_rows)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = t >> 4;
    const int part_i = (int)(t & 15);
    if (row >= n_rows) return;
    const half8_t v = *(const half8_t*)(q + row * kD + part_i * 8);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s = fmaf((float)v[e], (float)v[e], s);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row_max) {
        if (part_i == 0) {
            nq_out[row] = sqrtf(s);
            c_out[row] = row_max[row] * kLog2e + log2f(row_sum[row]);
        }
        return;
    }
    // the 16 lanes of the group share the KS partial (reference, sum) pairs, then combine
    float m = kNegBig, l = 0.f;
    for (int i = part_i; i < KS; i += 16) {
        const float2 ml = *(const float2*)(part + (row * KS + i) * 2);
        const float mn = fmaxf(m, ml.x);
        l = l * exp2f(m - mn) + ml.y * exp2f(ml.x - mn);
        m = mn;
    }
    float mg = m;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) mg = fmaxf(mg, __shfl_xor(mg, off, 64));
    l *= exp2f(m - mg);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) l += __shfl_xor(l, off, 64);
    if (part_i == 0) {
        nq_out[row] = sqrtf(s);
        c_out[row] = mg + log2f(l);
    }
}

// -------------------------------------------------------------------------------------------------
// phase 2: column reduction.  grid = (key blocks of 256, B*Hkv); each of the 8 waves owns 32 keys.
// Software-pipelined by one step: while the VALU rebuilds and reduces the probabilities of step t, the
// matrix pipe already computes the scores of step t+1, so the staged Q tiles run one step ahead of
// their row statistics (rings of three).
// -------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAsThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void ans_col_reduce(
    const half_t* __restrict__ q, const half_t* __restrict__ k, int64_t N, int64_t Nq, float c1,
    const float* __restrict__ c_row, const float* __restrict__ nq_row, float* __restrict__ ans_k,
    float* __restrict__ ans_v, int Hq, int Hkv, int G)
{
    __shared__ __attribute__((aligned(16))) half_t s_q[3][kTileHalfs];     // query tiles of steps t+1, t+2 (and t, spent)
    __shared__ __attribute__((aligned(16))) float s_c[3][32], s_n[3][32];  // row statistics of steps t, t+1, t+2
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, kh = lane >> 5;
    const int b = blockIdx.y / Hkv, g = blockIdx.y % Hkv;
    const int64_t kblk0 = (int64_t)blockIdx.x * 256;
    const int64_t k0 = kblk0 + wave * 32;                       // first key of this wave
    const int64_t key = k0 + n;
    const int64_t krow = key < N ? key : N - 1;
    Tile128 tk;
    load_tile(tk, k + (((int64_t)b * Hkv + g) * N + krow) * kD, kh);
    wait_all_loads();
    // first query tile that can see a key of this block:  N - Nq + i >= kblk0
    int64_t i_first = kblk0 - (N - Nq);
    if (i_first < 0) i_first = 0;
    i_first &= ~(int64_t)31;
    const int n_qt = (int)((Nq - i_first + 31) >> 5);           // query tiles per head
    const int n_steps = n_qt * G;                                // step = (head of the group, query tile)
    const int srow = tid >> 4, schunk = tid & 15;
    // (head, tile) of a step are tracked incrementally: no division in the loop
    auto fetch = [&](int hh, int qt, float& c_o, float& n_o) -> uint4_t {
        const int64_t i0 = i_first + (int64_t)qt * 32;
        const int64_t rbase = ((int64_t)b * Hq + g * G + hh) * Nq;
        const int64_t qrow = (i0 + srow < Nq) ? i0 + srow : Nq - 1;
        if (tid < 32) {
            const bool ok = i0 + tid < Nq;
            c_o = ok ? c_row[rbase + i0 + tid] : 3.0e38f;       // exp2(-huge) = 0 for rows past the end
            n_o = ok ? nq_row[rbase + i0 + tid] : 0.f;
        }
        return *(const uint4_t*)(q + (rbase + qrow) * kD + 8 * schunk);
    };
    auto stage = [&](int slot, const uint4_t& d, float c_o, float n_o) {
        *(uint4_t*)(&s_q[slot][srow * kRowPad + 8 * schunk]) = d;
        if (tid < 32) { s_c[slot][tid] = c_o; s_n[slot][tid] = n_o; }
    };
    int qt_f = 0, hh_f = 0;                                      // next step to fetch
    for (int i = 0; i < 2 && i < n_steps; ++i) {
        float c_o = 0.f, n_o = 0.f;
        const uint4_t d = fetch(hh_f, qt_f, c_o, n_o);
        stage(i, d, c_o, n_o);
        if (++qt_f == n_qt) { qt_f = 0; ++hh_f; }
    }
    __syncthreads();
    float16_t acc_cur;
    if (n_steps > 0) acc_cur = tile_dot_lds_a(s_q[0], tk, n, kh);   // rows = queries, cols = keys
    double sum_v = 0.0, sum_k = 0.0;
    int slot = 0, qt = 0;                                        // ring slot and query tile of the current step
    const int rel0 = (int)(N - Nq + i_first - k0);               // position of tile 0's first query minus this wave's first key
    for (int step = 0; step < n_steps; ++step) {
        const bool more = step + 2 < n_steps;
        uint4_t nxt = {0u, 0u, 0u, 0u};
        float c_o = 0.f, n_o = 0.f;
        if (more) nxt = fetch(hh_f, qt_f, c_o, n_o);
        const int s1 = slot == 2 ? 0 : slot + 1, s2 = s1 == 2 ? 0 : s1 + 1;
        const int rel = rel0 + 32 * qt;                          // (position of the tile's first query) - k0
        const int lim = n - rel;                                 // tile row r sees this lane's key iff r >= lim
        float pv = 0.f, pk = 0.f;
        float16_t acc_next;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_next[r] = 0.f;
        // scores of step t+1 (slot s1; past the last step the slot holds stale data and the result is dropped)
        // interleaved in program order with the reduction of step t, two elements per MFMA
        auto body = [&](auto masked) {
            float4_t c4 = {0.f, 0.f, 0.f, 0.f}, n4 = {0.f, 0.f, 0.f, 0.f};
            const half_t* ap = &s_q[s1][n * kRowPad + 8 * kh];
            half8_t a_op[8];
            a_op[0] = *(const half8_t*)(ap);
            a_op[1] = *(const half8_t*)(ap + 16);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                if (s + 2 < 8) a_op[s + 2] = *(const half8_t*)(ap + 16 * (s + 2));   // operand reads run two MFMAs ahead
                acc_next = __builtin_amdgcn_mfma_f32_32x32x16_f16(a_op[s], tk.v[s], acc_next, 0, 0, 0);
                const int qd = s >> 1;
                const int rl = 8 * qd + 4 * kh;                  // tile rows rl .. rl+3 live in acc[4qd .. 4qd+3]
                if ((s & 1) == 0) {
                    c4 = *(const float4_t*)(&s_c[slot][rl]);
                    n4 = *(const float4_t*)(&s_n[slot][rl]);
                }
#pragma unroll
                for (int e2 = 0; e2 < 2; ++e2) {
                    const int e = 2 * (s & 1) + e2;
                    float arg = fmaf(acc_cur[4 * qd + e], c1, -c4[e]);
                    if (decltype(masked)::value && rl + e < lim) arg = -3.0e38f;   // causal mask
                    const float a_ij = fast_exp2(arg);
                    pv += a_ij;
                    pk = fmaf(a_ij, fmaf(-a_ij, n4[e], n4[e]), pk);               // a (1 - a) ||q||
                }
            }
        };
        // only tiles on or above the diagonal (some query cannot see some key) pay for the mask; the branch is uniform
        if (__builtin_expect(rel < 31, 0)) body(std::true_type{});
        else body(std::false_type{});
        sum_v += (double)pv;
        sum_k += (double)pk;
        if (more) {
            stage(s2, nxt, c_o, n_o);
            if (++qt_f == n_qt) { qt_f = 0; ++hh_f; }
        }
        __syncthreads();
        acc_cur = acc_next;
        slot = s1;
        if (++qt == n_qt) qt = 0;
    }
    // lanes l and l+32 hold complementary query rows of the same key
    const double ov = __shfl_xor(sum_v, 32, 64), ok = __shfl_xor(sum_k, 32, 64);
    if (kh == 0 && key < N) {
        const int64_t o = ((int64_t)b * Hkv + g) * N + key;
        ans_v[o] = (float)(sum_v + ov);
        ans_k[o] = (float)(sum_k + ok);
    }
}

struct AsPlan {
    int KS;
    int64_t keys_per_split;
    size_t off_part, off_c, off_nq, off_ans_k, off_ans_v, total;
};

AsPlan plan(const Geom& g, int64_t N, int64_t Nq)
{
    AsPlan p;
    const int qspan = 32 * (8 / (g.G >= 4 ? 4 : g.G));          // query rows per workgroup of phase 1
    const int64_t qblocks = (Nq + qspan - 1) / qspan;
    const int64_t base_wgs = (int64_t)g.B * g.Hkv * qblocks;
    int64_t ks = (1024 + base_wgs - 1) / base_wgs;
    const int64_t max_ks = (N + 4095) / 4096;
    if (ks > max_ks) ks = max_ks;
    if (ks < 1) ks = 1;
    int64_t per = (N + ks - 1) / ks;
    per = (per + 31) / 32 * 32;
    p.keys_per_split = per;
    p.KS = (int)((N + per - 1) / per);
    const size_t rows = (size_t)g.B * g.Hq * Nq;
    size_t off = 0;
    p.off_part = off; off += align_up(rows * p.KS * 2 * sizeof(float));
    p.off_c = off;    off += align_up(rows * sizeof(float) + 16);
    p.off_nq = off;   off += align_up(rows * sizeof(float) + 16);
    p.off_ans_k = off; off += align_up((size_t)g.B * g.Hkv * N * sizeof(float));
    p.off_ans_v = off; off += align_up((size_t)g.B * g.Hkv * N * sizeof(float));
    p.total = off;
    return p;
}

}  // namespace

size_t anchor_score_workspace_bytes(const Geom& g, int64_t N, int64_t Nq) { return plan(g, N, Nq).total; }

// ans_k / ans_v may be NULL: the scores then live in the workspace at the offsets of the plan.
hipError_t launch_anchor_score(const Geom& g, const half_t* q, const half_t* k, int64_t N, int64_t Nq, float scale,
                               const float* row_max, const float* row_sum, float* ans_k, float* ans_v, void* ws,
                               hipStream_t st)
{
    const AsPlan p = plan(g, N, Nq);
    char* w = (char*)ws;
    float* part = (float*)(w + p.off_part);
    float* c_row = (float*)(w + p.off_c);
    float* nq_row = (float*)(w + p.off_nq);
    if (!ans_k) ans_k = (float*)(w + p.off_ans_k);
    if (!ans_v) ans_v = (float*)(w + p.off_ans_v);
    const float c1 = scale * kLog2e;
    const int64_t rows = (int64_t)g.B * g.Hq * Nq;
    if (!row_max) {
        const int qspan = 32 * (8 / (g.G >= 4 ? 4 : g.G));
        dim3 grid((unsigned)p.KS, (unsigned)((Nq + qspan - 1) / qspan), (unsigned)(g.B * g.Hkv));
        hipLaunchKernelGGL(ans_row_stats, grid, dim3(kAsThreads), 0, st, q, k, N, Nq, c1, part, g.Hq, g.Hkv, g.G,
                           p.KS, p.keys_per_split);
    }
    hipLaunchKernelGGL(ans_finalize_stats, dim3((unsigned)((rows * 16 + 255) / 256)), dim3(256), 0, st, q, part, p.KS,
                       row_max, row_sum, c_row, nq_row, rows);
    dim3 grid2((unsigned)((N + 255) / 256), (unsigned)(g.B * g.Hkv));
    hipLaunchKernelGGL(ans_col_reduce, grid2, dim3(kAsThreads), 0, st, q, k, N, Nq, c1, c_row, nq_row, ans_k, ans_v,
                       g.Hq, g.Hkv, g.G);
    return hipGetLastError();
}

}  // namespace antkv
