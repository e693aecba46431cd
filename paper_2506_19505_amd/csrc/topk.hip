// Top-k selection of Anchor Scores (keep the ~1 % highest-scoring tokens in FP16; paper Sec. 3,
// Fig. 2(b)) and the gather of the selected FP16 rows.
//
// Exact radix select on an order-preserving 32-bit key:
//   1. histogram of the top 11 key bits per row;
//   2. every workgroup (slice of 8192 scores) finds the bin d0 that holds the k-th largest key and counts its keys in
//      higher bins.  If bin d0 holds few keys (at most N/8 + 4096, the usual case for heavy-tailed scores) the
//      workgroup appends its keys of that bin, with their positions, to the row's candidate list; otherwise (scores
//      crowded into a narrow range) it adds them to a second histogram over the next 11 bits;
//   3. only for rows that took the second branch: the same once more, one level down (count the keys of bin d0
//      above the second digit d1, list the keys with prefix (d0, d1)); workgroups of other rows return at once;
//   4. one workgroup per row selects the exact k-th largest key tau among the candidates (radix rounds on the
//      remaining bits, histograms in LDS) and adds the candidates' share to the per-slice counts of keys > tau and
//      == tau; a row whose keys agree in 22 bits for more than the list holds is walked by that workgroup instead;
//   5. an ordered emission pass writes the positions of all keys > tau plus the lowest-positioned keys == tau
//      needed to reach k, in ascending position order.
#include "common.h"

namespace antkv {

namespace {

constexpr int kSlice = 8192;
constexpr int kTopkThreads = 256;
constexpr int kBins = kTopkBins;

// Find the bin where the count of keys taken from the top reaches k_rem.
// On return digit = that bin, k_new = how many keys are still needed inside it.
template <int THREADS = kTopkThreads>
__device__ void find_digit(const uint32_t* __restrict__ hist, int nbins, uint32_t k_rem,
                           uint32_t& digit, uint32_t& k_new, uint32_t* sh)   // sh: 2 + THREADS / 64 words
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bpt = nbins / THREADS;
    uint32_t c[kBins / THREADS];
    uint32_t tot = 0;
    for (int i = 0; i < bpt; ++i) {
        c[i] = hist[nbins - 1 - (tid * bpt + i)];
        tot += c[i];
    }
    uint32_t incl = tot;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t n = __shfl_up(incl, off, 64);
        if (lane >= off) incl += n;
    }
    if (lane == 63) sh[2 + wave] = incl;
    __syncthreads();
    uint32_t prefix = incl - tot;
    for (int w = 0; w < wave; ++w) prefix += sh[2 + w];
    for (int i = 0; i < bpt; ++i) {
        if (prefix < k_rem && prefix + c[i] >= k_rem) {
            sh[0] = (uint32_t)(nbins - 1 - (tid * bpt + i));
            sh[1] = k_rem - prefix;
        }
        prefix += c[i];
    }
    __syncthreads();
    digit = sh[0];
    k_new = sh[1];
    __syncthreads();
}

__global__ __launch_bounds__(256) void zero_u32(uint32_t* p, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__device__ __forceinline__ const float* row_scores(const float* scores, const float* scores_b, int rows_a, int64_t row,
                                                   int64_t N)
{
    return (row < rows_a) ? scores + row * N : scores_b + (row - rows_a) * N;
}

// per-row header in the workspace
enum { kHeadCount = 0, kHeadTau = 1, kHeadNeedEq = 2, kHeadWords = 8 };

__global__ __launch_bounds__(kTopkThreads) void topk_hist0(const float* __restrict__ scores,
                                                           const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                           uint32_t* __restrict__ ws_hist)
{
    __shared__ uint32_t lh[kBins];
    const int64_t row = blockIdx.y;
    for (int i = threadIdx.x; i < kBins; i += kTopkThreads) lh[i] = 0u;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * kSlice;
    const int64_t hi = (lo + kSlice < N) ? lo + kSlice : N;
    const float* src = row_scores(scores, scores_b, rows_a, row, N);
    if (hi - lo == kSlice && (((uintptr_t)(src + lo)) & 15) == 0) {
#pragma unroll
        for (int j = 0; j < kSlice / (4 * kTopkThreads); ++j) {
            const float4_t v = *(const float4_t*)(src + lo + 4 * (threadIdx.x + kTopkThreads * j));
#pragma unroll
            for (int e = 0; e < 4; ++e) atomicAdd(&lh[float_key(v[e]) >> 21], 1u);
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kTopkThreads) atomicAdd(&lh[float_key(src[i]) >> 21], 1u);
    }
    __syncthreads();
    uint32_t* hist = ws_hist + row * 2 * kBins;
    for (int i = threadIdx.x; i < kBins; i += kTopkThreads)
        if (lh[i]) atomicAdd(&hist[i], lh[i]);
}

// LEVEL 1: per slice, count the keys above bin d0; list the keys of bin d0, or (crowded bin) histogram their next
// 11 bits.  LEVEL 2, rows with a crowded bin only: count the keys of bin d0 above the second digit d1 and list the
// keys with prefix (d0, d1).
template <int LEVEL>
__global__ __launch_bounds__(kTopkThreads) void topk_collect(const float* __restrict__ scores,
                                                             const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                             uint32_t k, uint32_t* __restrict__ ws_hist,
                                                             uint32_t* __restrict__ head, uint32_t* __restrict__ counts,
                                                             int n_slices, uint2_t* __restrict__ cand, uint32_t cap)
{
    __shared__ uint32_t lh[LEVEL == 1 ? kBins : 1];
    __shared__ uint32_t sh[8];
    __shared__ uint32_t red[2][4];
    __shared__ uint32_t s_base;
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t* hist0 = ws_hist + row * 2 * kBins;
    uint32_t* hist1 = hist0 + kBins;
    uint32_t d0, k_rem;
    find_digit(hist0, kBins, k, d0, k_rem, sh);
    const bool crowded = hist0[d0] > cap;                       // the same for every workgroup of the row
    uint32_t prefix = d0;                                       // keys that match it are the candidates of this level
    bool list = !crowded;
    if (LEVEL == 2) {
        if (!crowded) return;
        uint32_t d1;
        find_digit(hist1, kBins, k_rem, d1, k_rem, sh);
        prefix = (d0 << 11) | d1;
        list = hist1[d1] <= cap;
    }
    constexpr int kShift = LEVEL == 1 ? 21 : 10;
    if (LEVEL == 1 && crowded) {
        for (int i = tid; i < kBins; i += kTopkThreads) lh[i] = 0u;
        __syncthreads();
    }
    const int64_t lo = (int64_t)blockIdx.x * kSlice;
    const int64_t hi = (lo + kSlice < N) ? lo + kSlice : N;
    const float* src = row_scores(scores, scores_b, rows_a, row, N);
    constexpr int kPer = kSlice / kTopkThreads;                 // 32 scores per thread, in 8 groups of 4
    uint32_t key[kPer];
    const bool fast = hi - lo == kSlice && (((uintptr_t)(src + lo)) & 15) == 0;
    // element j of the thread sits at position lo + pos(j)
    auto pos = [&](int j) -> int64_t {
        return fast ? 4 * (tid + kTopkThreads * (j >> 2)) + (j & 3) : (int64_t)tid + (int64_t)kTopkThreads * j;
    };
    if (fast) {
#pragma unroll
        for (int j = 0; j < kPer / 4; ++j) {
            const float4_t v = *(const float4_t*)(src + lo + 4 * (tid + kTopkThreads * j));
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = float_key(v[e]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPer; ++j) key[j] = (lo + pos(j) < hi) ? float_key(src[lo + pos(j)]) : 0u;
    }
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const bool in = fast || lo + pos(j) < hi;
        const uint32_t p = key[j] >> kShift;
        // LEVEL 2 counts only keys of bin d0 (higher bins were counted by LEVEL 1)
        gt += in && p > prefix && (LEVEL == 1 || (key[j] >> 21) == d0);
        eq += in && p == prefix;
    }
    // block-wide: total of gt, exclusive prefix of eq
    uint32_t ieq = eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(ieq, off, 64);
        if (lane >= off) ieq += a;
    }
    gt = wave_sum_u32(gt);
    if (lane == 63) red[1][wave] = ieq;
    if (lane == 0) red[0][wave] = gt;
    __syncthreads();
    uint32_t off_eq = ieq - eq;
    for (int w = 0; w < wave; ++w) off_eq += red[1][w];
    const uint32_t tot_eq = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    if (tid == 0) {
        uint32_t* c = counts + (row * n_slices + blockIdx.x) * 2;
        const uint32_t tot_gt = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        if (LEVEL == 1) { c[0] = tot_gt; c[1] = 0u; }
        else c[0] += tot_gt;                                    // this workgroup owns its slice's counters
        s_base = (list && tot_eq) ? atomicAdd(&head[row * kHeadWords + kHeadCount], tot_eq) : 0u;
    }
    __syncthreads();
    if (list) {
        if (eq == 0) return;
        uint32_t at = s_base + off_eq;
        uint2_t* out = cand + row * (int64_t)cap;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const bool in = fast || lo + pos(j) < hi;
            if (in && (key[j] >> kShift) == prefix) {
                if (at < cap) out[at] = uint2_t{key[j], (uint32_t)(lo + pos(j))};
                ++at;
            }
        }
    } else if (LEVEL == 1) {                                    // crowded bin: its next 11 bits go to the second histogram
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const bool in = fast || lo + pos(j) < hi;
            if (in && (key[j] >> 21) == d0) atomicAdd(&lh[(key[j] >> 10) & 2047u], 1u);
        }
        __syncthreads();
        for (int i = tid; i < kBins; i += kTopkThreads)
            if (lh[i]) atomicAdd(&hist1[i], lh[i]);
    }
}

// per row: exact k-th largest key among the candidates, and the candidates' share of the per-slice counts
constexpr int kResolveThreads = 1024;

__global__ __launch_bounds__(kResolveThreads) void topk_resolve(const float* __restrict__ scores,
                                                             const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                             uint32_t k, const uint32_t* __restrict__ ws_hist,
                                                             uint32_t* __restrict__ head, uint32_t* __restrict__ counts,
                                                             int n_slices, const uint2_t* __restrict__ cand, uint32_t cap)
{
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t lh_eq[kBins];
    __shared__ uint32_t sh[2 + kResolveThreads / 64];
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const uint32_t* hist0 = ws_hist + row * 2 * kBins;
    const uint32_t* hist1 = hist0 + kBins;
    uint32_t d0, d1 = 0, d2, k_rem, need_eq;
    find_digit<kResolveThreads>(hist0, kBins, k, d0, k_rem, sh);
    const bool crowded = hist0[d0] > cap;
    uint32_t n_cand = hist0[d0];
    bool listed = true;
    if (crowded) {
        find_digit<kResolveThreads>(hist1, kBins, k_rem, d1, k_rem, sh);
        n_cand = hist1[d1];
        listed = n_cand <= cap;                                  // else more than the list holds agree in 22 bits: walk the row
    }
    const uint32_t prefix22 = (d0 << 11) | d1;
    const uint2_t* list = cand + row * (int64_t)cap;
    const float* src = row_scores(scores, scores_b, rows_a, row, N);
    auto for_each = [&](auto fn) {
        if (listed) {
            for (uint32_t i = tid; i < n_cand; i += kResolveThreads) fn(list[i][0], list[i][1]);
        } else {
            for (int64_t i = tid; i < N; i += kResolveThreads) {
                const uint32_t key = float_key(src[i]);
                if ((key >> 10) == prefix22) fn(key, (uint32_t)i);
            }
        }
    };
    if (!crowded) {                                              // the candidates share d0 only: round on bits 20..10
        for (int i = tid; i < kBins; i += kResolveThreads) lh[i] = 0u;
        __syncthreads();
        for_each([&](uint32_t key, uint32_t) { atomicAdd(&lh[(key >> 10) & 2047u], 1u); });
        __syncthreads();
        find_digit<kResolveThreads>(lh, kBins, k_rem, d1, k_rem, sh);
    }
    for (int i = tid; i < kBins; i += kResolveThreads) lh[i] = 0u;
    __syncthreads();
    for_each([&](uint32_t key, uint32_t) { if (((key >> 10) & 2047u) == d1) atomicAdd(&lh[key & 1023u], 1u); });
    __syncthreads();
    find_digit<kResolveThreads>(lh, 1024, k_rem, d2, need_eq, sh);
    const uint32_t tau = (d0 << 21) | (d1 << 10) | d2;
    // the candidates' share of the per-slice counts.  Thousands of candidates fall into a few slices, so they are
    // counted in LDS first (one global add per slice afterwards) whenever the row has at most 2048 slices.
    uint32_t* c = counts + row * (int64_t)n_slices * 2;
    if (n_slices <= kBins) {
        __syncthreads();
        for (int i = tid; i < kBins; i += kResolveThreads) { lh[i] = 0u; lh_eq[i] = 0u; }
        __syncthreads();
        for_each([&](uint32_t key, uint32_t i) {
            if (key > tau) atomicAdd(&lh[i / kSlice], 1u);
            else if (key == tau) atomicAdd(&lh_eq[i / kSlice], 1u);
        });
        __syncthreads();
        for (int i = tid; i < n_slices; i += kResolveThreads) {    // this workgroup is the only writer of the row's counts now
            if (lh[i]) c[i * 2] += lh[i];
            if (lh_eq[i]) c[i * 2 + 1] += lh_eq[i];
        }
    } else {
        for_each([&](uint32_t key, uint32_t i) {
            if (key > tau) atomicAdd(&c[(i / kSlice) * 2], 1u);
            else if (key == tau) atomicAdd(&c[(i / kSlice) * 2 + 1], 1u);
        });
    }
    if (tid == 0) {
        head[row * kHeadWords + kHeadTau] = tau;
        head[row * kHeadWords + kHeadNeedEq] = need_eq;
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_emit(const float* __restrict__ scores,
                                                          const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                          uint32_t k, const uint32_t* __restrict__ head,
                                                          const uint32_t* __restrict__ counts, int n_slices,
                                                          int32_t* __restrict__ idx, int32_t* __restrict__ idx_b)
{
    __shared__ uint32_t red[2][4];
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t tau = head[row * kHeadWords + kHeadTau], need_eq = head[row * kHeadWords + kHeadNeedEq];
    // keys > tau and == tau in the slices before this one
    uint32_t bgt = 0, beq = 0;
    for (int s = tid; s < (int)blockIdx.x; s += kTopkThreads) {
        bgt += counts[(row * n_slices + s) * 2];
        beq += counts[(row * n_slices + s) * 2 + 1];
    }
    bgt = wave_sum_u32(bgt);
    beq = wave_sum_u32(beq);
    if (lane == 0) { red[0][wave] = bgt; red[1][wave] = beq; }
    __syncthreads();
    const uint32_t base_gt = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    const uint32_t base_eq = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    __syncthreads();
    // each thread owns 32 consecutive scores of the slice
    const int64_t lo = (int64_t)blockIdx.x * kSlice + (int64_t)tid * (kSlice / kTopkThreads);
    int64_t hi = lo + kSlice / kTopkThreads;
    if (hi > N) hi = N;
    const float* src = row_scores(scores, scores_b, rows_a, row, N);
    // the thread's 32 scores are read once (16-byte loads when the row allows it) and kept as keys
    constexpr int kPer = kSlice / kTopkThreads;
    static_assert(kPer == 32, "a thread owns 32 consecutive scores");
    uint32_t key[kPer];
    const int n_own = (hi > lo) ? (int)(hi - lo) : 0;
    if (n_own == kPer && (((uintptr_t)(src + lo)) & 15) == 0) {
#pragma unroll
        for (int j = 0; j < kPer / 4; ++j) {
            const float4_t v = *(const float4_t*)(src + lo + 4 * j);
#pragma unroll
            for (int e = 0; e < 4; ++e) key[4 * j + e] = float_key(v[e]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < kPer; ++j) key[j] = (j < n_own) ? float_key(src[lo + j]) : 0u;
    }
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        gt += (j < n_own) && (key[j] > tau);
        eq += (j < n_own) && (key[j] == tau);
    }
    uint32_t igt = gt, ieq = eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t a = __shfl_up(igt, off, 64), b = __shfl_up(ieq, off, 64);
        if (lane >= off) { igt += a; ieq += b; }
    }
    if (lane == 63) { red[0][wave] = igt; red[1][wave] = ieq; }
    __syncthreads();
    uint32_t run_gt = base_gt + igt - gt, run_eq = base_eq + ieq - eq;
    for (int w = 0; w < wave; ++w) { run_gt += red[0][w]; run_eq += red[1][w]; }
    int32_t* out = (row < rows_a) ? idx + row * (int64_t)k : idx_b + (row - rows_a) * (int64_t)k;
    if (gt == 0 && (eq == 0 || run_eq >= need_eq)) return;       // nothing of this thread is selected
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        if (j < n_own) {
            if (key[j] > tau) {
                out[run_gt + (run_eq < need_eq ? run_eq : need_eq)] = (int32_t)(lo + j);
                ++run_gt;
            } else if (key[j] == tau) {
                if (run_eq < need_eq) out[run_gt + run_eq] = (int32_t)(lo + j);
                ++run_eq;
            }
        }
    }
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4_t* __restrict__ x, int64_t N,
                                                          const int32_t* __restrict__ idx, int64_t k,
                                                          uint4_t* __restrict__ rows, int64_t n_items)
{
    // one 16-lane group per row of 128 fp16 = 16 x 16 B
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t item = t >> 4;
    const int part = (int)(t & 15);
    if (item >= n_items) return;
    const int64_t bg = item / k;
    const int64_t j = idx[item];
    rows[item * 16 + part] = x[(bg * N + j) * 16 + part];
}

}  // namespace

namespace {

struct TopkPlan {
    int n_slices;
    uint32_t cap;                      // candidate entries per row
    size_t off_hist, off_head, off_counts, off_cand, total;
};

TopkPlan topk_plan(int64_t rows, int64_t N)
{
    TopkPlan p;
    p.n_slices = (int)((N + kSlice - 1) / kSlice);
    if (p.n_slices < 1) p.n_slices = 1;
    // the bin of the k-th key usually holds a few percent of a row; a fuller bin makes topk_resolve walk the row
    p.cap = (uint32_t)(N / 8 + 4096);
    size_t off = 0;
    p.off_hist = off;   off += align_up((size_t)rows * 2 * kBins * 4);            // two histogram levels per row
    p.off_head = off;   off += align_up((size_t)rows * kHeadWords * 4);     // directly after the histograms: zeroed together
    p.off_counts = off; off += align_up((size_t)rows * p.n_slices * 2 * 4);
    p.off_cand = off;   off += align_up((size_t)rows * p.cap * sizeof(uint2_t));
    p.total = off;
    return p;
}

}  // namespace

size_t topk_workspace_bytes(int64_t n_rows, int64_t N, int64_t k)
{
    (void)k;
    return topk_plan(n_rows, N).total;
}

// Two score arrays of n_rows rows each can be selected in one go (scores_b / idx_b may be NULL): the launches then
// cover 2 n_rows rows, the first n_rows from `scores` into `idx`, the rest from `scores_b` into `idx_b`.
namespace {

// clears the histograms and headers of `rows` rows
uint32_t* topk_clear(int64_t rows, int64_t N, void* ws, hipStream_t st)
{
    const TopkPlan p = topk_plan(rows, N);
    uint32_t* hist = (uint32_t*)((char*)ws + p.off_hist);
    const int64_t nz = (int64_t)(p.off_counts / 4);             // histograms and headers
    hipLaunchKernelGGL(zero_u32, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, hist, nz);
    return hist;
}

// everything after the first-level histogram
hipError_t topk_select(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                       int64_t N, int64_t k, void* ws, hipStream_t st)
{
    const int64_t rows = scores_b ? 2 * n_rows : n_rows;
    const TopkPlan p = topk_plan(rows, N);
    char* w = (char*)ws;
    uint32_t* hist = (uint32_t*)(w + p.off_hist);
    uint32_t* head = (uint32_t*)(w + p.off_head);
    uint32_t* counts = (uint32_t*)(w + p.off_counts);
    uint2_t* cand = (uint2_t*)(w + p.off_cand);
    const int ra = (int)n_rows;
    dim3 grid(p.n_slices, (unsigned)rows);
    hipLaunchKernelGGL(topk_collect<1>, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist, head,
                       counts, p.n_slices, cand, p.cap);
    hipLaunchKernelGGL(topk_collect<2>, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist, head,
                       counts, p.n_slices, cand, p.cap);
    hipLaunchKernelGGL(topk_resolve, dim3((unsigned)rows), dim3(kResolveThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k,
                       hist, head, counts, p.n_slices, cand, p.cap);
    hipLaunchKernelGGL(topk_emit, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, head, counts,
                       p.n_slices, idx, idx_b);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_topk2(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                        int64_t N, int64_t k, void* ws, hipStream_t st)
{
    if (k == 0 || n_rows == 0) return hipSuccess;
    const int64_t rows = scores_b ? 2 * n_rows : n_rows;
    uint32_t* hist = topk_clear(rows, N, ws, st);
    const TopkPlan p = topk_plan(rows, N);
    dim3 grid(p.n_slices, (unsigned)rows);
    hipLaunchKernelGGL(topk_hist0, grid, dim3(kTopkThreads), 0, st, scores, scores_b, (int)n_rows, N, hist);
    return topk_select(scores, idx, scores_b, idx_b, n_rows, N, k, ws, st);
}

uint32_t* launch_topk2_begin(int64_t n_rows, int64_t N, void* ws, hipStream_t st) { return topk_clear(2 * n_rows, N, ws, st); }

hipError_t launch_topk2_finish(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                               int64_t N, int64_t k, void* ws, hipStream_t st)
{
    if (k == 0 || n_rows == 0) return hipSuccess;
    return topk_select(scores, idx, scores_b, idx_b, n_rows, N, k, ws, st);
}

hipError_t launch_topk(const float* scores, int64_t n_rows, int64_t N, int64_t k, int32_t* idx, void* ws,
                       hipStream_t st)
{
    return launch_topk2(scores, idx, nullptr, nullptr, n_rows, N, k, ws, st);
}

hipError_t launch_gather_rows(const Geom& g, const half_t* x, int64_t N, const int32_t* idx, int64_t k,
                              half_t* rows, hipStream_t st)
{
    const int64_t n_items = (int64_t)g.B * g.Hkv * k;
    if (n_items == 0) return hipSuccess;
    const int64_t threads = n_items * 16;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                       (const uint4_t*)x, N, idx, k, (uint4_t*)rows, n_items);
    return hipGetLastError();
}

}  // namespace antkv
