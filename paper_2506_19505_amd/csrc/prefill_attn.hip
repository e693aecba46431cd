// Causal attention over the prompt (paper Sec. 2.1) that also writes the softmax row statistics which the
// Anchor Score pass consumes (Alg. 1, first step: attention extended to return row maximum and row sum).
//
// grid = (query blocks, B*Hkv); 8 waves = HG heads of the group x 8/HG query tiles of 32, HG = min(G, 4), so that
// every wave has work whatever the group size (4 x 2, 2 x 4 or 1 x 8; larger groups loop over the heads).
// The waves of a workgroup share each 32-key tile of K and V through double-buffered LDS.
//   scores   S^T tile (keys on the MFMA row axis, queries on the column axis): lane (n, kh) owns query n and
//            16 of the tile's 32 keys, so the running softmax is lane-local up to one exchange between the two
//            half-waves, which must share the reference because their products meet in one accumulator.
//   output   O^T += V^T P^T, again with queries on the column axis: the B operand is the lane's own 16
//            probabilities (fp16), the A operand comes out of the V tile through ds_read_b64_tr_b16, and the
//            accumulator rows of a lane all belong to its query, so a moved reference rescales registers only.
// Probabilities are exp2 against a per-query reference that trails the running maximum: it moves only when a
// tile brings a score more than kPMax (log2 units) above it, which keeps fp16 P below 2^kPMax.
#include "common.h"

#include <type_traits>

namespace antkv {

namespace {

constexpr int kPaThreads = 512;
constexpr int kKRow = 136;      // halfs per staged K row: 16-byte reads of 16 consecutive rows hit 16 bank quads
constexpr int kVRow = 160;      // halfs per staged V row (320 B): the 4 rows x 64 bytes that two 16-lane blocks read in one pass hit 64 banks
constexpr float kPMax = 12.f;

typedef __attribute__((address_space(3))) short4_t lds_short4;

__device__ __forceinline__ half4_t read_tr16(const half_t* p)
{
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)p);
    return __builtin_bit_cast(half4_t, v);
}

__global__ __launch_bounds__(kPaThreads) void prefill_attn_kernel(
    const half_t* __restrict__ q, const half_t* __restrict__ k, const half_t* __restrict__ v, int64_t N, int64_t Nq,
    float c1, half_t* __restrict__ out, float* __restrict__ row_max, float* __restrict__ row_sum, int Hq, int Hkv, int G)
{
    __shared__ __attribute__((aligned(16))) half_t s_k[2][32 * kKRow];
    __shared__ __attribute__((aligned(16))) half_t s_v[2][32 * kVRow];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // scalar, so that per-wave conditions are scalar branches
    const int n = lane & 31, kh = lane >> 5;
    const int64_t qblk = (int64_t)gridDim.x - 1 - blockIdx.x;      // longest rows first
    const int b = blockIdx.y / Hkv, g = blockIdx.y % Hkv;
    const int HG = G >= 4 ? 4 : G;                                 // head slots of the workgroup
    const int qspan = 32 * (8 / HG);                               // query rows per workgroup
    const int64_t q0 = qblk * qspan + (wave >> (HG >> 1)) * 32;
    const bool wave_on = q0 < Nq;
    const int64_t qi = q0 + n;
    const int64_t qrow = qi < Nq ? qi : Nq - 1;
    const int64_t qpos = N - Nq + qrow;                            // last key this lane's query sees
    const int64_t tile_last_pos = N - Nq + ((q0 + 31 < Nq) ? q0 + 31 : Nq - 1);
    const int64_t blk_last_pos = N - Nq + ((qblk * qspan + qspan - 1 < Nq) ? qblk * qspan + qspan - 1 : Nq - 1);
    const int64_t k_end = blk_last_pos + 1;                        // keys the workgroup walks
    const int64_t k_hi = tile_last_pos + 1;                        // keys this wave needs
    const half_t* kbase = k + ((int64_t)b * Hkv + g) * N * kD;
    const half_t* vbase = v + ((int64_t)b * Hkv + g) * N * kD;
    const int srow = tid >> 4, schunk = tid & 15;                  // staging: 16 bytes per thread and tile
    // transposed V reads: inside a 16-lane block, lane 4e + c reads key row e, channels 4c .. 4c+3; blocks 0/1
    // cover the two channel halves of a 32-channel group, blocks 2/3 the same for the other key half (kh)
    const int tr_off = (4 * kh + ((lane & 15) >> 2)) * kVRow + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    for (int h_it = 0; h_it < (G + HG - 1) / HG; ++h_it) {
        const int hh = HG * h_it + (wave & (HG - 1));
        const bool head_on = wave_on && hh < G;
        const int h = g * G + (hh < G ? hh : G - 1);
        half8_t tq[8];
        {
            const half_t* qp = q + (((int64_t)b * Hq + h) * Nq + qrow) * kD;
#pragma unroll
            for (int s = 0; s < 8; ++s) tq[s] = *(const half8_t*)(qp + 16 * s + 8 * kh);
#pragma unroll
            for (int s = 0; s < 8; ++s) pin(tq[s]);
            wait_all_loads();
        }
        float16_t o[4];
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[cg][r] = 0.f;
        float m_ref = kNegBig, m_true = kNegBig, l_run = 0.f;
        int buf = 0;
        auto fetch_k = [&](int64_t kt) -> uint4_t {
            const int64_t row = (kt + srow < N) ? kt + srow : N - 1;
            return *(const uint4_t*)(kbase + row * kD + 8 * schunk);
        };
        auto fetch_v = [&](int64_t kt) -> uint4_t {
            const int64_t row = (kt + srow < N) ? kt + srow : N - 1;
            return *(const uint4_t*)(vbase + row * kD + 8 * schunk);
        };
        *(uint4_t*)(&s_k[0][srow * kKRow + 8 * schunk]) = fetch_k(0);
        *(uint4_t*)(&s_v[0][srow * kVRow + 8 * schunk]) = fetch_v(0);
        __syncthreads();
        for (int64_t kt = 0; kt < k_end; kt += 32) {
            const bool more = kt + 32 < k_end;
            uint4_t nk = {0u, 0u, 0u, 0u}, nv = {0u, 0u, 0u, 0u};
            if (more) { nk = fetch_k(kt + 32); nv = fetch_v(kt + 32); }
            if (head_on && kt < k_hi) {
                float16_t acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const half8_t a = *(const half8_t*)(&s_k[buf][n * kKRow + 16 * s + 8 * kh]);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, tq[s], acc, 0, 0, 0);   // rows = keys, cols = queries
                }
                const bool init = m_ref > kNegBig;
                const float base = init ? m_ref : 0.f;
                float p[16];
                float mx = kNegBig;
                const int lim = (int)(qpos - kt);                  // key offset <= lim is visible
                auto scores = [&](auto masked) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float x = fmaf(acc[r], c1, -base);
                        if (decltype(masked)::value && 8 * (r >> 2) + 4 * kh + (r & 3) > lim) x = kNegBig;
                        p[r] = x;
                        mx = fmaxf(mx, x);
                    }
                };
                // only tiles on the causal diagonal pay for the mask; the branch is uniform
                if (__builtin_expect(kt + 31 <= N - Nq + q0, 1)) scores(std::false_type{});
                else scores(std::true_type{});
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));            // the two key halves of a query agree on the reference
                const bool seen = mx > 0.5f * kNegBig;
                if (seen) m_true = fmaxf(m_true, base + mx);
                if (seen && !(init && mx <= kPMax)) {              // move the reference to this tile's maximum
                    const float alpha = init ? fast_exp2(-mx) : 0.f;
                    l_run *= alpha;
#pragma unroll
                    for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[cg][r] *= alpha;
#pragma unroll
                    for (int r = 0; r < 16; ++r) p[r] -= mx;
                    m_ref = base + mx;
                }
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    p[r] = fast_exp2(p[r]);
                    sum += p[r];
                }
                l_run += sum;
                // O^T += V^T P^T: k-slot j of half kh in step s is key 16s + 8(j>>2) + 4kh + (j&3), on both operands
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    half8_t pb;
#pragma unroll
                    for (int j = 0; j < 8; ++j) pb[j] = (half_t)p[8 * s + j];
#pragma unroll
                    for (int cg = 0; cg < 4; ++cg) {
                        const half_t* vp = &s_v[buf][tr_off + 16 * s * kVRow + 32 * cg];
                        const half4_t a0 = read_tr16(vp), a1 = read_tr16(vp + 8 * kVRow);
                        const half8_t a = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
                        o[cg] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pb, o[cg], 0, 0, 0);   // rows = channels
                    }
                }
            }
            if (more) {
                *(uint4_t*)(&s_k[buf ^ 1][srow * kKRow + 8 * schunk]) = nk;
                *(uint4_t*)(&s_v[buf ^ 1][srow * kVRow + 8 * schunk]) = nv;
            }
            __syncthreads();
            buf ^= 1;
        }
        const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
        if (head_on && qi < Nq) {
            const int64_t row = ((int64_t)b * Hq + h) * Nq + qi;
            const float inv = 1.f / l_tot;
            half_t* op = out + row * kD + 4 * kh;
#pragma unroll
            for (int cg = 0; cg < 4; ++cg)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {                  // accumulator rows 8qd + 4kh + e = channels of group cg
                    half4_t w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (half_t)(o[cg][4 * qd + e] * inv);
                    *(half4_t*)(op + 32 * cg + 8 * qd) = w;
                }
            if (kh == 0 && row_max) {
                row_max[row] = m_true * (1.f / kLog2e);
                row_sum[row] = l_tot * fast_exp2(m_ref - m_true);
            }
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_prefill_attn(const Geom& g, const half_t* q, const half_t* k, const half_t* v, int64_t N, int64_t Nq,
                               float scale, half_t* out, float* row_max, float* row_sum, hipStream_t st)
{
    const int qspan = 32 * (8 / (g.G >= 4 ? 4 : g.G));
    dim3 grid((unsigned)((Nq + qspan - 1) / qspan), (unsigned)(g.B * g.Hkv));
    hipLaunchKernelGGL(prefill_attn_kernel, grid, dim3(kPaThreads), 0, st, q, k, v, N, Nq, scale * kLog2e, out, row_max,
                       row_sum, g.Hq, g.Hkv, g.G);
    return hipGetLastError();
}

}  // namespace antkv
