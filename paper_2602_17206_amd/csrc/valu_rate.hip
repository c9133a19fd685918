// Micro-benchmark of the vector-ALU figures the DP sweeps are priced against on gfx950:
//   (1) issue rate per SIMD of the instructions a DP step consists of, with 1, 2 and 4 wavefronts
//       per SIMD (8 independent chains per wavefront),
//   (2) latency of the same instructions in one dependent chain,
//   (3) the DP step itself (Sec. 2 Eq. 1-2: soft-minimum of three neighbours plus the cost, with the
//       lane shift that brings the neighbouring row's value), as one wavefront runs it: cycles per
//       step with 1, 2 and 4 such wavefronts per SIMD.
// Not part of the library: a stand-alone program, built next to it.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#include "kernels.h"
#include "dp_kernels.h"

#define CHECK(x)                                                                        \
    do {                                                                                \
        hipError_t e_ = (x);                                                            \
        if (e_ != hipSuccess) {                                                         \
            printf("hip error %s at line %d\n", hipGetErrorString(e_), __LINE__);       \
            exit(1);                                                                    \
        }                                                                               \
    } while (0)

enum { ADD_F32, FMA_F32, ADD_F64, MIN_F64, FMA_F64, EXP_F32, LOG_F32, CVT_F32_F64, CVT_F64_F32, MOV_DPP };

template <int OP> __device__ __forceinline__ void one(double &a, const double &a2, float &f, const float &f2)
{
    if (OP == ADD_F32) asm volatile("v_add_f32 %0, %0, %1" : "+v"(f) : "v"(f2));
    if (OP == FMA_F32) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(f) : "v"(f2));
    if (OP == ADD_F64) asm volatile("v_add_f64 %0, %0, %1" : "+v"(a) : "v"(a2));
    if (OP == MIN_F64) asm volatile("v_min_f64 %0, %0, %1" : "+v"(a) : "v"(a2));
    if (OP == FMA_F64) asm volatile("v_fma_f64 %0, %0, %1, %0" : "+v"(a) : "v"(a2));
    if (OP == EXP_F32) asm volatile("v_exp_f32 %0, %0" : "+v"(f));
    if (OP == LOG_F32) asm volatile("v_log_f32 %0, %0" : "+v"(f));
    if (OP == CVT_F32_F64) asm volatile("v_cvt_f32_f64 %0, %1" : "=v"(f) : "v"(a));
    if (OP == CVT_F64_F32) asm volatile("v_cvt_f64_f32 %0, %1" : "=v"(a) : "v"(f));
    if (OP == MOV_DPP) asm volatile("v_mov_b32_dpp %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(f) : "v"(f2));
}

// 8 independent chains: 32 instructions per iteration
template <int OP> __global__ void rate_kernel(double *out, int iters)
{
    double a[8];
    float f[8];
    for (int i = 0; i < 8; ++i) {
        a[i] = threadIdx.x * 1e-3 + i;
        f[i] = threadIdx.x * 1e-3f + i;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i) one<OP>(a[i], a[(i + 1) & 7], f[i], f[(i + 1) & 7]);
    }
    double s = 0;
    for (int i = 0; i < 8; ++i) s += a[i] + f[i];
    if (s == 12345.678) out[0] = s;
}

// one dependent chain: 32 instructions per iteration
template <int OP> __global__ void latency_kernel(double *out, int iters)
{
    double a = threadIdx.x * 1e-3, b = 1.0000001;
    float f = threadIdx.x * 1e-3f, g = 1.0001f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 32; ++r) one<OP>(a, b, f, g);
    }
    if (a + f == 12345.678) out[0] = a;
}

// the DP step, 32 steps per iteration, costs and the row above from registers
__global__ void dp_step_kernel(double *out, int iters, double c2d)
{
    const int lane = threadIdx.x & 63;
    double left = sdtw::kBig, diag = lane == 0 ? 0.0 : sdtw::kBig;
    float dc[8];
    for (int i = 0; i < 8; ++i) dc[i] = 0.25f * ((lane * 7 + i * 3) & 15) + 0.5f;
    const double top = 3.0 + lane;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = sdtw::lane_shr1(left, top);
            double m;
            float L;
            sdtw::softmin3_parts(diag, up, left, m, L);
            const double cur = fma((double)dc[u & 7], c2d, m) - (double)L;
            diag = up;
            left = cur;
        }
    }
    if (left == 12345.678) out[0] = left;
}

// the same step with the memory traffic of the real consumer added piece by piece:
//   bit 0: cost read from an LDS ring, bit 1: the value written to LDS for the neighbouring band,
//   bit 2: the value stored to the table in HBM (non-temporal, one 512-byte row per step),
//   bit 3: one workgroup barrier per 32 steps, with two more wavefronts that only take the barrier
template <int V> __global__ __launch_bounds__(192) void dp_step_mem_kernel(double *table, int iters, double c2d)
{
    __shared__ float ring[64 * 129];
    __shared__ double eo[64 + 32];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int e = threadIdx.x; e < 64 * 129; e += blockDim.x) ring[e] = 0.25f * (e & 15) + 0.5f;
    __syncthreads();
    if (w > 0) {
        if (V & 8)
            for (int it = 0; it < iters; ++it) __syncthreads();
        return;
    }
    double left = sdtw::kBig, diag = lane == 0 ? 0.0 : sdtw::kBig;
    float dc[8];
    for (int i = 0; i < 8; ++i) dc[i] = 0.25f * ((lane * 7 + i * 3) & 15) + 0.5f;
    const double top = 3.0 + lane;
    const float *my_ring = ring + lane * 129;
    double *my_eo = eo + (lane == 63 ? 0 : 32 + lane);
    double *Rk = table + (size_t)blockIdx.x * 4 * 32 * 64;  // 4 macro-steps of table per workgroup, rewritten
    for (int it = 0; it < iters; ++it) {
        const float *rd = my_ring + (it & 3) * 32;
        double *Rs = Rk + (size_t)(it & 3) * 32 * 64;
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = sdtw::lane_shr1(left, top);
            const float d = (V & 1) ? rd[u] : dc[u & 7];
            double m;
            float L;
            sdtw::softmin3_parts(diag, up, left, m, L);
            const double cur = fma((double)d, c2d, m) - (double)L;
            if (V & 4) __builtin_nontemporal_store(cur, &Rs[u * 64 + lane]);
            if (V & 2) my_eo[u & 31] = cur;
            diag = up;
            left = cur;
        }
        if (V & 8) __syncthreads();
    }
    if (left == 12345.678) table[0] = left;
}

// Does matrix-core work of another wavefront on the same SIMD slow the DP step down?  Wavefronts 0-3
// of a workgroup (one per SIMD) run the DP step; wavefronts 4-7 (same SIMDs) run `mfma_per_32_steps`
// dependent v_mfma_f32_32x32x16_f16 per 32 steps' worth of iterations (0: they only exist), or, with
// FP32_PARTNER, a chain of float32 additions instead of the DP step.
template <bool FP32_PARTNER> __global__ __launch_bounds__(512) void coexec_kernel(double *out, int iters, int mfma_per_iter, double c2d)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (w >= 4) {
        sdtw::half8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * (lane + i)); b[i] = (_Float16)(0.002f * (lane - i)); }
        sdtw::floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it)
            for (int m = 0; m < mfma_per_iter; ++m) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
        if (acc[0] == 12345.678f) out[1] = acc[3];
        return;
    }
    if (FP32_PARTNER) {
        float f = lane * 1e-3f, g = 1.0001f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 32 * 19; ++u) asm volatile("v_add_f32 %0, %0, %1" : "+v"(f) : "v"(g));
        }
        if (f == 12345.678f) out[0] = f;
        return;
    }
    double left = sdtw::kBig, diag = lane == 0 ? 0.0 : sdtw::kBig;
    float dc[8];
    for (int i = 0; i < 8; ++i) dc[i] = 0.25f * ((lane * 7 + i * 3) & 15) + 0.5f;
    const double top = 3.0 + lane;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = sdtw::lane_shr1(left, top);
            double m;
            float L;
            sdtw::softmin3_parts(diag, up, left, m, L);
            const double cur = fma((double)dc[u & 7], c2d, m) - (double)L;
            diag = up;
            left = cur;
        }
    }
    if (left == 12345.678) out[0] = left;
}

static float timed(void (*launch)(int, int, double *), int waves_per_simd, int iters, double *d)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch(waves_per_simd, 10, d);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    launch(waves_per_simd, iters, d);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    return ms;
}

template <int OP> static void launch_rate(int w, int iters, double *d) { rate_kernel<OP><<<256, 256 * w>>>(d, iters); }
template <int OP> static void launch_lat(int, int iters, double *d) { latency_kernel<OP><<<256, 256>>>(d, iters); }
static void launch_dp(int w, int iters, double *d) { dp_step_kernel<<<256, 256 * w>>>(d, iters, 14.4); }
static int g_mfma = 0;
template <bool F> static void launch_coexec(int, int iters, double *d) { coexec_kernel<F><<<256, 512>>>(d, iters, g_mfma, 14.4); }
static double *g_table = nullptr;
template <int V> static void launch_mem(int, int iters, double *) { dp_step_mem_kernel<V><<<256, 192>>>(g_table, iters, 14.4); }

int main()
{
    double *d;
    CHECK(hipMalloc(&d, 64));
    const int iters = 2000;
    const double ghz = 2.4;  // nominal; the clock under load may be lower, ratios are what matters
    struct Row { const char *name; void (*rate)(int, int, double *); void (*lat)(int, int, double *); };
    const Row rows[] = {
        {"v_add_f32", launch_rate<ADD_F32>, launch_lat<ADD_F32>},     {"v_fma_f32", launch_rate<FMA_F32>, launch_lat<FMA_F32>},
        {"v_add_f64", launch_rate<ADD_F64>, launch_lat<ADD_F64>},     {"v_min_f64", launch_rate<MIN_F64>, launch_lat<MIN_F64>},
        {"v_fma_f64", launch_rate<FMA_F64>, launch_lat<FMA_F64>},     {"v_exp_f32", launch_rate<EXP_F32>, launch_lat<EXP_F32>},
        {"v_log_f32", launch_rate<LOG_F32>, launch_lat<LOG_F32>},     {"v_cvt_f32_f64", launch_rate<CVT_F32_F64>, nullptr},
        {"v_cvt_f64_f32", launch_rate<CVT_F64_F32>, nullptr},         {"v_mov_b32_dpp", launch_rate<MOV_DPP>, launch_lat<MOV_DPP>},
    };
    printf("cycles at %.1f GHz per instruction per SIMD (1 workgroup per CU, 4*w wavefronts)\n", ghz);
    printf("%-16s %10s %10s %10s %12s\n", "instruction", "w=1", "w=2", "w=4", "dependent");
    for (const Row &r : rows) {
        printf("%-16s", r.name);
        for (int w = 1; w <= 4; w *= 2)
            printf(" %10.2f", timed(r.rate, w, iters, d) * 1e-3 * ghz * 1e9 / ((double)iters * 32 * w));
        if (r.lat) printf(" %12.2f", timed(r.lat, 1, iters, d) * 1e-3 * ghz * 1e9 / ((double)iters * 32));
        printf("\n");
        fflush(stdout);
    }
    printf("DP step (soft-minimum of three + cost, one wavefront = 64 rows): cycles at %.1f GHz per step\n", ghz);
    for (int w = 1; w <= 4; w *= 2) {
        const double cyc = timed(launch_dp, w, iters, d) * 1e-3 * ghz * 1e9 / ((double)iters * 32);
        printf("  %d wavefront(s) per SIMD: %.1f per step of one wavefront, %.1f per step per SIMD\n", w, cyc, cyc / w);
        fflush(stdout);
    }
    printf("DP step of one wavefront with a matrix-core wavefront on the same SIMD (v_mfma_f32_32x32x16_f16 per 32 steps):\n");
    for (int m : {0, 12, 24, 48, 96}) {
        g_mfma = m;
        const double dp = timed(launch_coexec<false>, 1, iters / 4, d) * 1e-3 * ghz * 1e9 / ((double)(iters / 4) * 32);
        const double f32 = timed(launch_coexec<true>, 1, iters / 4, d) * 1e-3 * ghz * 1e9 / ((double)(iters / 4) * 32);
        printf("  %3d MFMA per 32 steps: DP step %.1f cycles; 19 dependent float32 additions instead: %.1f cycles\n", m, dp, f32);
        fflush(stdout);
    }
    CHECK(hipMalloc(&g_table, (size_t)256 * 4 * 32 * 64 * sizeof(double)));
    printf("one wavefront per compute unit, the step with the consumer's memory traffic added: cycles per step\n");
    struct Var { const char *name; void (*fn)(int, int, double *); };
    const Var vars[] = {{"arithmetic only", launch_mem<0>}, {"+ cost from LDS", launch_mem<1>}, {"+ edge value to LDS", launch_mem<3>},
                        {"+ table store to HBM", launch_mem<7>}, {"+ barrier per 32 steps", launch_mem<15>},
                        {"table store only", launch_mem<4>}, {"barrier only", launch_mem<8>}};
    for (const Var &v : vars) {
        printf("  %-26s %.1f\n", v.name, timed(v.fn, 1, iters / 8, d) * 1e-3 * ghz * 1e9 / ((double)(iters / 8) * 32));
        fflush(stdout);
    }
    CHECK(hipFree(g_table));
    CHECK(hipFree(d));
    return 0;
}
