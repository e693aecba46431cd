// Micro-benchmarks of the MI355X (gfx950) limits that the decode-attention design is priced against.
// Standalone program (not part of libantkv.so): prints one line per probe.
//
//   hbm      streaming read rate over a buffer far larger than the 256 MB Infinity Cache
//   lds      LDS read rates per CU for the access shapes the decode kernel uses: 8-byte table gathers whose bank is
//            picked by the lane (conflict-free by construction) or by the data (random), 16-byte linear reads,
//            transposed 8-byte reads (ds_read_b64_tr_b16) with the two 16-lane blocks of an LDS pass on the same or
//            on different banks, and float atomics
//   issue    VALU and MFMA issue rates per SIMD, alone, interleaved inside a wave and split over the waves of a SIMD
//            (do the two pipes overlap?), and both together with LDS reads in flight
//
// Every kernel runs 256 workgroups of 1024 threads (one per CU, 4 waves per SIMD), like the decode kernel.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                                          \
    do {                                                                                               \
        hipError_t e_ = (x);                                                                           \
        if (e_ != hipSuccess) {                                                                        \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);                     \
            fflush(stdout);                                                                            \
            exit(1);                                                                                   \
        }                                                                                              \
    } while (0)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v lds_short4;
typedef __attribute__((address_space(3))) char lds_char;

static const int kCUs = 256;
static double g_clk_hz = 2.4e9;     // replaced by the measured shader clock

// ---------------------------------------------------------------------------------------- clock
__global__ void clock_probe(long long* out)
{
    const long long c0 = clock64(), w0 = wall_clock64();
    float x = threadIdx.x;
    for (int i = 0; i < 400000; ++i) x = fmaf(x, 0.999f, 0.01f);
    const long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; out[2] = (long long)x; }
}

// ---------------------------------------------------------------------------------------- HBM
__global__ __launch_bounds__(256) void hbm_read(const uint4v* __restrict__ src, size_t n16, uint32_t* out)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4v a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a[0] ^ a[3] ^ b[1] ^ b[2] ^ c[0] ^ c[3] ^ d[1] ^ d[2];
    }
    if (acc == 0x12345678u) out[0] = acc;
}

// ---------------------------------------------------------------------------------------- LDS
// Pure LDS instruction streams: every lane keeps eight fixed addresses in registers and the loop is nothing but
// reads (inline assembly, results unused) and one wait per eight reads, so the figure is the LDS pipe's own rate.
// The table is 256 rows of 256 bytes (a row spans all 64 banks).
enum LdsMode {
    B64_DISTINCT,      // ds_read_b64: the 32 lanes of a pass on 32 different 8-byte slots, rows arbitrary (table gather)
    B64_TWO_WAY,       // ds_read_b64: the two 16-lane blocks of a pass on the same 32 banks (different rows)
    B64_RANDOM,        // ds_read_b64: slot and row arbitrary per lane
    B128_LINEAR,       // ds_read_b128: consecutive 16-byte pieces
    B128_ROWS,         // ds_read_b128: 16 lanes cover a 256-byte row, rows arbitrary
    TR_DISTINCT,       // ds_read_b64_tr_b16 with the B64_DISTINCT addresses
    TR_TWO_WAY,        // ds_read_b64_tr_b16 with the B64_TWO_WAY addresses
    B32_LINEAR,        // ds_read_b32: consecutive dwords
    W32_LINEAR,        // ds_write_b32: consecutive dwords
    W64_LINEAR,        // ds_write_b64
    ATOMIC_F32         // ds_add_f32, a different bank per lane
};

__device__ __forceinline__ uint32_t mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <int MODE>
__global__ __launch_bounds__(1024) void lds_probe(uint32_t* out, int iters)
{
    extern __shared__ uint4v smem[];
    uint32_t* s32 = (uint32_t*)smem;
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) s32[i] = (MODE == ATOMIC_F32) ? 0u : i * 2654435761u;
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t base = (uint32_t)(uintptr_t)(const lds_char*)smem;
    uint32_t ad[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const uint32_t r = mix(threadIdx.x * 8u + u + 1u);
        const uint32_t row = r & 255u;
        uint32_t a;
        if (MODE == B64_DISTINCT || MODE == TR_DISTINCT) a = (row << 8) | ((lane & 31u) << 3);
        else if (MODE == B64_TWO_WAY || MODE == TR_TWO_WAY) a = (row << 8) | ((lane & 15u) << 3);
        else if (MODE == B64_RANDOM) a = (row << 8) | (((r >> 8) & 31u) << 3);
        else if (MODE == B128_LINEAR) a = ((uint32_t)u * 1024u + lane * 16u);
        else if (MODE == B128_ROWS) a = (row << 8) | ((lane & 15u) << 4);
        else if (MODE == B32_LINEAR || MODE == W32_LINEAR) a = ((uint32_t)u * 256u + lane * 4u) + ((threadIdx.x >> 6) << 11);
        else if (MODE == W64_LINEAR) a = ((uint32_t)u * 512u + lane * 8u) + ((threadIdx.x >> 6) << 12);
        else a = (row << 8) | (lane << 2);
        ad[u] = base + (a & 65535u);
    }
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        if (MODE == B64_DISTINCT || MODE == B64_TWO_WAY || MODE == B64_RANDOM) {
            uint2v r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b64 %0, %8\n ds_read_b64 %1, %9\n ds_read_b64 %2, %10\n ds_read_b64 %3, %11\n"
                         "ds_read_b64 %4, %12\n ds_read_b64 %5, %13\n ds_read_b64 %6, %14\n ds_read_b64 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
            acc |= r0[0] & r7[1] & 1u;
        } else if (MODE == TR_DISTINCT || MODE == TR_TWO_WAY) {
            uint2v r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b64_tr_b16 %0, %8\n ds_read_b64_tr_b16 %1, %9\n ds_read_b64_tr_b16 %2, %10\n ds_read_b64_tr_b16 %3, %11\n"
                         "ds_read_b64_tr_b16 %4, %12\n ds_read_b64_tr_b16 %5, %13\n ds_read_b64_tr_b16 %6, %14\n ds_read_b64_tr_b16 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
            acc |= r0[0] & r7[1] & 1u;
        } else if (MODE == B128_LINEAR || MODE == B128_ROWS) {
            uint4v r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
                         "ds_read_b128 %4, %12\n ds_read_b128 %5, %13\n ds_read_b128 %6, %14\n ds_read_b128 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
            acc |= r0[0] & r7[3] & 1u;
        } else if (MODE == B32_LINEAR) {
            uint32_t r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b32 %0, %8\n ds_read_b32 %1, %9\n ds_read_b32 %2, %10\n ds_read_b32 %3, %11\n"
                         "ds_read_b32 %4, %12\n ds_read_b32 %5, %13\n ds_read_b32 %6, %14\n ds_read_b32 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
            acc |= r0 & r7 & 1u;
        } else if (MODE == W32_LINEAR) {
            asm volatile("ds_write_b32 %0, %8\n ds_write_b32 %1, %8\n ds_write_b32 %2, %8\n ds_write_b32 %3, %8\n"
                         "ds_write_b32 %4, %8\n ds_write_b32 %5, %8\n ds_write_b32 %6, %8\n ds_write_b32 %7, %8\n"
                         "s_waitcnt lgkmcnt(0)"
                         :: "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]), "v"(acc)
                         : "memory");
        } else if (MODE == W64_LINEAR) {
            const uint2v val = {acc, lane};
            asm volatile("ds_write_b64 %0, %8\n ds_write_b64 %1, %8\n ds_write_b64 %2, %8\n ds_write_b64 %3, %8\n"
                         "ds_write_b64 %4, %8\n ds_write_b64 %5, %8\n ds_write_b64 %6, %8\n ds_write_b64 %7, %8\n"
                         "s_waitcnt lgkmcnt(0)"
                         :: "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]), "v"(val)
                         : "memory");
        } else {
            const float one = 1.0f;
            asm volatile("ds_add_f32 %0, %8\n ds_add_f32 %1, %8\n ds_add_f32 %2, %8\n ds_add_f32 %3, %8\n"
                         "ds_add_f32 %4, %8\n ds_add_f32 %5, %8\n ds_add_f32 %6, %8\n ds_add_f32 %7, %8\n"
                         "s_waitcnt lgkmcnt(0)"
                         :: "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]), "v"(one)
                         : "memory");
        }
    }
    if (acc == 0x12345678u) out[0] = acc;
}

// ---------------------------------------------------------------------------------------- issue
// Per loop iteration a wave issues NM MFMAs and NV VALU instructions.  split = 0: every wave does both, interleaved
// one MFMA per NV / NM VALU (the scheduler barriers keep that order); split = 1: the waves of a SIMD alternate roles.
// KIND: 0 = v_mfma_f32_16x16x32_f16, 1 = v_mfma_i32_16x16x64_i8, 2 = v_smfmac_f32_16x16x64_f16,
// 3 = v_smfmac_f32_32x32x32_f16 (two accumulators).  LDS = 1 adds one
// conflict-free 8-byte LDS read per 4 VALU instructions.
template <int KIND, int NM, int NV, int LDS>
__global__ __launch_bounds__(1024) void issue_probe(float* out, int iters, int split)
{
    extern __shared__ uint4v smem[];
    if (LDS) {
        uint32_t* s32 = (uint32_t*)smem;
        for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) s32[i] = i;
        __syncthreads();
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    half8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(lane * 0.001f + i); b[i] = (_Float16)(lane * 0.002f - i); }
    half16 b16;
    for (int i = 0; i < 16; ++i) b16[i] = (_Float16)(lane * 0.002f - i);
    int4v ia = {lane, lane + 1, lane + 2, lane + 3}, ib = {lane * 3, lane * 5, lane * 7, lane * 9};
    float4v c[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    int4v ci[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    float16v cw[2] = {};
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = lane + i;
    uint32_t lacc = 0;
    const bool do_m = !split || ((wave >> 2) & 1) == 0;      // waves w, w+4, w+8, w+12 share a SIMD: roles alternate
    const bool do_v = !split || ((wave >> 2) & 1) == 1;
    constexpr int VPM = NM > 0 ? NV / NM : NV;
    for (int it = 0; it < iters; ++it) {
        if (split) {
            if (do_m) {
#pragma unroll
                for (int u = 0; u < NM; ++u) {
                    if (KIND == 0) c[u & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c[u & 3], 0, 0, 0);
                    else if (KIND == 1) ci[u & 3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ia, ib, ci[u & 3], 0, 0, 0);
                    else if (KIND == 2) c[u & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, b16, c[u & 3], 0x4444, 0, 0);
                    else cw[u & 1] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, cw[u & 1], 0x4444, 0, 0);
                }
            }
            if (do_v) {
#pragma unroll
                for (int u = 0; u < NV; ++u) v[u & 7] = __builtin_fmaf(v[u & 7], 1.0001f, 0.5f);
            }
        } else {
#pragma unroll
            for (int u = 0; u < (NM > 0 ? NM : 1); ++u) {
                if (NM > 0) {
                    if (KIND == 0) c[u & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c[u & 3], 0, 0, 0);
                    else if (KIND == 1) ci[u & 3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ia, ib, ci[u & 3], 0, 0, 0);
                    else if (KIND == 2) c[u & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, b16, c[u & 3], 0x4444, 0, 0);
                    else cw[u & 1] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, cw[u & 1], 0x4444, 0, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one MFMA ...
                }
#pragma unroll
                for (int k = 0; k < VPM; ++k) {
                    v[k & 7] = __builtin_fmaf(v[k & 7], 1.0001f, 0.5f);
                    if (LDS && (k & 3) == 0) {
                        const uint2v r = *(const uint2v*)((const char*)smem + ((((uint32_t)(it + u + k) & 255u) << 8) | ((uint32_t)(lane & 31) << 3)));
                        lacc ^= r[0] ^ r[1];
                    }
                }
                if (NM > 0) __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);  // ... then its share of the VALU work
            }
        }
    }
    float s = (float)lacc;
    for (int i = 0; i < 8; ++i) s += v[i];
    for (int i = 0; i < 4; ++i) s += c[i][0] + (float)ci[i][0];
    s += cw[0][0] + cw[1][5];
    out[blockIdx.x * 1024 + threadIdx.x] = s;
}

template <typename F>
static float time_ms(F f, int reps)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    f();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) f();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / reps;
}

template <int MODE>
static void run_lds(const char* name, uint32_t* out, int bytes_per_lane)
{
    const int iters = 4000;
    CK(hipFuncSetAttribute((const void*)lds_probe<MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    const float ms = time_ms([&] { hipLaunchKernelGGL((lds_probe<MODE>), dim3(kCUs), dim3(1024), 65536, 0, out, iters); }, 5);
    const double wave_instr = 16.0 * iters * 8;                          // wave-level LDS instructions per CU
    const double clk = ms * 1e-3 * g_clk_hz;
    printf("lds  %-62s %8.3f ms  %6.2f clk per wave instruction per CU  %7.1f B/clk/CU\n", name, ms, clk / wave_instr,
           wave_instr * 64 * bytes_per_lane / clk);
    fflush(stdout);
}

template <int KIND, int NM, int NV, int LDS>
static void run_issue(const char* name, float* out, int split)
{
    const int iters = 4000;
    CK(hipFuncSetAttribute((const void*)issue_probe<KIND, NM, NV, LDS>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
    const float ms = time_ms([&] { hipLaunchKernelGGL((issue_probe<KIND, NM, NV, LDS>), dim3(kCUs), dim3(1024), 65536, 0, out, iters, split); }, 3);
    const double clk_per_iter = ms * 1e-3 * g_clk_hz / iters;           // SIMD clocks per loop iteration (4 waves per SIMD)
    printf("issue %-58s %8.3f ms  %7.1f clk per iteration per SIMD\n", name, ms, clk_per_iter);
    fflush(stdout);
}

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    printf("device %s  CUs %d  LDS per workgroup %zu\n", prop.name, prop.multiProcessorCount, prop.sharedMemPerBlock);
    uint32_t* out;
    CK(hipMalloc(&out, 256 * 1024 * 4));
    {
        long long* d;
        CK(hipMalloc(&d, 64));
        hipLaunchKernelGGL(clock_probe, dim3(1), dim3(64), 0, 0, d);
        hipLaunchKernelGGL(clock_probe, dim3(1), dim3(64), 0, 0, d);
        long long h[3];
        CK(hipMemcpy(h, d, 24, hipMemcpyDeviceToHost));
        g_clk_hz = (double)h[0] / ((double)h[1] / 100e6);
        printf("clock: %.0f MHz shader clock (clock64 against the 100 MHz wall clock, one busy wave)\n", g_clk_hz / 1e6);
        CK(hipFree(d));
    }
    {
        const size_t bytes = (size_t)4 << 30;
        uint4v* src;
        CK(hipMalloc(&src, bytes));
        CK(hipMemset(src, 1, bytes));
        for (int grid : {2048, 4096, 8192}) {
            const float ms = time_ms([&] { hipLaunchKernelGGL(hbm_read, dim3(grid), dim3(256), 0, 0, src, bytes / 16, out); }, 5);
            printf("hbm  read 4 GiB, %5d workgroups of 256 %30s %8.3f ms  %7.1f GB/s\n", grid, "", ms, bytes / (ms * 1e-3) / 1e9);
            fflush(stdout);
        }
        CK(hipFree(src));
    }
    run_lds<B64_DISTINCT>("ds_read_b64, a pass on 32 different slots, rows arbitrary", out, 8);
    run_lds<B64_TWO_WAY>("ds_read_b64, the two blocks of a pass on the same 32 banks", out, 8);
    run_lds<B64_RANDOM>("ds_read_b64, slot and row arbitrary", out, 8);
    run_lds<B128_LINEAR>("ds_read_b128, consecutive", out, 16);
    run_lds<B128_ROWS>("ds_read_b128, 16 lanes per 256-byte row, rows arbitrary", out, 16);
    run_lds<TR_DISTINCT>("ds_read_b64_tr_b16, a pass on 32 different slots", out, 8);
    run_lds<TR_TWO_WAY>("ds_read_b64_tr_b16, the two blocks of a pass on the same 32 banks", out, 8);
    run_lds<B32_LINEAR>("ds_read_b32, consecutive", out, 4);
    run_lds<W32_LINEAR>("ds_write_b32, consecutive", out, 4);
    run_lds<W64_LINEAR>("ds_write_b64, consecutive", out, 8);
    run_lds<ATOMIC_F32>("ds_add_f32, a different bank per lane", out, 4);

    float* fo = (float*)out;
    run_issue<0, 0, 128, 0>("128 VALU fma", fo, 0);
    run_issue<0, 16, 0, 0>("16 MFMA f16 16x16x32", fo, 0);
    run_issue<1, 16, 0, 0>("16 MFMA i8 16x16x64", fo, 0);
    run_issue<2, 16, 0, 0>("16 sparse MFMA f16 16x16x64", fo, 0);
    run_issue<3, 16, 0, 0>("16 sparse MFMA f16 32x32x32", fo, 0);
    run_issue<3, 16, 128, 0>("16 sparse MFMA 32x32x32 + 128 VALU, interleaved in every wave", fo, 0);
    run_issue<0, 16, 128, 0>("16 MFMA f16 + 128 VALU, interleaved in every wave", fo, 0);
    run_issue<1, 16, 128, 0>("16 MFMA i8 + 128 VALU, interleaved in every wave", fo, 0);
    run_issue<2, 16, 128, 0>("16 sparse MFMA + 128 VALU, interleaved in every wave", fo, 0);
    run_issue<0, 16, 64, 0>("16 MFMA f16 + 64 VALU, interleaved in every wave", fo, 0);
    run_issue<0, 16, 128, 0>("16 MFMA f16 | 128 VALU, roles split over the waves", fo, 1);
    run_issue<0, 0, 128, 1>("128 VALU + 32 LDS reads", fo, 0);
    run_issue<0, 16, 128, 1>("16 MFMA f16 + 128 VALU + 32 LDS reads, interleaved", fo, 0);
    printf("done\n");
    return 0;
}
