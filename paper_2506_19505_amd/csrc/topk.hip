// Top-k selection of Anchor Scores (keep the ~1 % highest-scoring tokens in FP16; paper Sec. 3,
// Fig. 2(b)) and the gather of the selected FP16 rows.
//
// Exact radix select on an order-preserving 32-bit key: three histogram passes (11 + 11 + 10 bits)
// find the k-th largest key tau; one counting pass and one ordered emission pass then write the
// positions of all keys > tau plus the lowest-positioned keys == tau needed to reach k, in
// ascending position order.  Rows are split into slices of 8192 scores so that a launch has
// (slices x rows) workgroups; every workgroup re-derives tau's known digits from the global
// histograms itself, so no extra "scan" launches are needed.
#include "common.h"

namespace antkv {

namespace {

constexpr int kSlice = 8192;
constexpr int kTopkThreads = 256;
constexpr int kBins = 2048;

// Find the bin where the count of keys taken from the top reaches k_rem.
// On return digit = that bin, k_new = how many keys are still needed inside it.
__device__ void find_digit(const uint32_t* __restrict__ hist, int nbins, uint32_t k_rem,
                           uint32_t& digit, uint32_t& k_new, uint32_t* sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bpt = nbins / kTopkThreads;
    uint32_t c[kBins / kTopkThreads];
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

template <int PASS>
__global__ __launch_bounds__(kTopkThreads) void topk_hist(const float* __restrict__ scores,
                                                          const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                          uint32_t k, uint32_t* __restrict__ ws_hist)
{
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t sh[8];
    const int64_t row = blockIdx.y;
    uint32_t* hist = ws_hist + row * 3 * kBins;
    for (int i = threadIdx.x; i < kBins; i += kTopkThreads) lh[i] = 0u;
    uint32_t prefix = 0, k_rem = k;
    if (PASS >= 1) {
        uint32_t d0;
        find_digit(hist, kBins, k_rem, d0, k_rem, sh);
        prefix = d0;
    }
    if (PASS >= 2) {
        uint32_t d1;
        find_digit(hist + kBins, kBins, k_rem, d1, k_rem, sh);
        prefix = (prefix << 11) | d1;
    }
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * kSlice;
    const int64_t hi = (lo + kSlice < N) ? lo + kSlice : N;
    const float* src = (row < rows_a) ? scores + row * N : scores_b + (row - rows_a) * N;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kTopkThreads) {
        const uint32_t key = float_key(src[i]);
        if (PASS == 0) atomicAdd(&lh[key >> 21], 1u);
        else if (PASS == 1) { if ((key >> 21) == prefix) atomicAdd(&lh[(key >> 10) & 2047u], 1u); }
        else { if ((key >> 10) == prefix) atomicAdd(&lh[key & 1023u], 1u); }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += kTopkThreads)
        if (lh[i]) atomicAdd(&hist[PASS * kBins + i], lh[i]);
}

__device__ void resolve_tau(const uint32_t* hist, uint32_t k, uint32_t& tau, uint32_t& need_eq, uint32_t* sh)
{
    uint32_t d0, d1, d2, k_rem = k;
    find_digit(hist, kBins, k_rem, d0, k_rem, sh);
    find_digit(hist + kBins, kBins, k_rem, d1, k_rem, sh);
    find_digit(hist + 2 * kBins, 1024, k_rem, d2, k_rem, sh);
    tau = (d0 << 21) | (d1 << 10) | d2;
    need_eq = k_rem;
}

// per slice: how many keys are > tau and == tau
__global__ __launch_bounds__(kTopkThreads) void topk_count(const float* __restrict__ scores,
                                                           const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                           uint32_t k, const uint32_t* __restrict__ ws_hist,
                                                           uint32_t* __restrict__ counts, int n_slices)
{
    __shared__ uint32_t sh[8];
    __shared__ uint32_t red[2][4];
    const int64_t row = blockIdx.y;
    uint32_t tau, need_eq;
    resolve_tau(ws_hist + row * 3 * kBins, k, tau, need_eq, sh);
    const int64_t lo = (int64_t)blockIdx.x * kSlice;
    const int64_t hi = (lo + kSlice < N) ? lo + kSlice : N;
    const float* src = (row < rows_a) ? scores + row * N : scores_b + (row - rows_a) * N;
    uint32_t gt = 0, eq = 0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kTopkThreads) {
        const uint32_t key = float_key(src[i]);
        gt += (key > tau);
        eq += (key == tau);
    }
    gt = wave_sum_u32(gt);
    eq = wave_sum_u32(eq);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = gt; red[1][threadIdx.x >> 6] = eq; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t* c = counts + (row * n_slices + blockIdx.x) * 2;
        c[0] = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        c[1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_emit(const float* __restrict__ scores,
                                                          const float* __restrict__ scores_b, int rows_a, int64_t N,
                                                          uint32_t k, const uint32_t* __restrict__ ws_hist,
                                                          const uint32_t* __restrict__ counts, int n_slices,
                                                          int32_t* __restrict__ idx, int32_t* __restrict__ idx_b)
{
    __shared__ uint32_t sh[8];
    __shared__ uint32_t red[2][4];
    const int64_t row = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t tau, need_eq;
    resolve_tau(ws_hist + row * 3 * kBins, k, tau, need_eq, sh);
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
    const float* src = (row < rows_a) ? scores + row * N : scores_b + (row - rows_a) * N;
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

size_t topk_workspace_bytes(int64_t n_rows, int64_t N, int64_t k)
{
    (void)k;
    const int64_t n_slices = (N + kSlice - 1) / kSlice;
    return align_up((size_t)n_rows * 3 * kBins * 4) + align_up((size_t)n_rows * (n_slices > 0 ? n_slices : 1) * 2 * 4);
}

// Two score arrays of n_rows rows each can be selected in one go (scores_b / idx_b may be NULL): the launches then
// cover 2 n_rows rows, the first n_rows from `scores` into `idx`, the rest from `scores_b` into `idx_b`.
hipError_t launch_topk2(const float* scores, int32_t* idx, const float* scores_b, int32_t* idx_b, int64_t n_rows,
                        int64_t N, int64_t k, void* ws, hipStream_t st)
{
    if (k == 0 || n_rows == 0) return hipSuccess;
    const int64_t rows = scores_b ? 2 * n_rows : n_rows;
    const int n_slices = (int)((N + kSlice - 1) / kSlice);
    uint32_t* hist = (uint32_t*)ws;
    uint32_t* counts = (uint32_t*)((char*)ws + align_up((size_t)rows * 3 * kBins * 4));
    const int64_t nh = rows * 3 * kBins;
    const int ra = (int)n_rows;
    hipLaunchKernelGGL(zero_u32, dim3((unsigned)((nh + 255) / 256)), dim3(256), 0, st, hist, nh);
    dim3 grid(n_slices, (unsigned)rows);
    hipLaunchKernelGGL(topk_hist<0>, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist);
    hipLaunchKernelGGL(topk_hist<1>, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist);
    hipLaunchKernelGGL(topk_hist<2>, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist);
    hipLaunchKernelGGL(topk_count, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist, counts, n_slices);
    hipLaunchKernelGGL(topk_emit, grid, dim3(kTopkThreads), 0, st, scores, scores_b, ra, N, (uint32_t)k, hist, counts, n_slices,
                       idx, idx_b);
    return hipGetLastError();
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
