// Calibration kernels behind sdtw_debug_rate_probe (a benchmark hook, not part of the hot path):
// the vector-ALU figures the DP sweeps are priced against on gfx950.
//   probe 0: issue rate of one instruction of the DP step, 8 independent chains per wavefront
//   probe 1: the same instruction in one dependent chain (latency)
//   probe 2: the bare DP step (Sec. 2 Eq. 1-2: soft-minimum of three neighbours plus the cost, with
//            the lane shift that brings the neighbouring row's value), one row per lane
//   probe 3: the bare DP step with TWO rows per lane (a 128-row band: lane t owns rows 2t and 2t+1,
//            at step s their cells (2t, s-2t) and (2t+1, s-2t-1) are independent of each other)
//   probe 4: the DP step of one wavefront per SIMD with a matrix-core wavefront on the same SIMD
//   probe 5: the DP step with the consumer's memory traffic added piece by piece
// Every kernel runs `iters` iterations of 32 instructions (probes 0, 1) or 32 steps (the others).
#pragma once
#include <hip/hip_runtime.h>

#include "device_core.h"
#include "dp_kernels.h"

namespace sdtw {
namespace probe {

enum { ADD_F32, FMA_F32, ADD_F64, MIN_F64, FMA_F64, EXP_F32, LOG_F32, CVT_F32_F64, CVT_F64_F32, MOV_DPP, kOps };

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

__device__ __forceinline__ void lane_costs(float (&dc)[8], int lane)
{
    for (int i = 0; i < 8; ++i) dc[i] = 0.25f * ((lane * 7 + i * 3) & 15) + 0.5f;
}

// the DP step, 32 steps per iteration, costs and the row above from registers
__global__ void dp_step_kernel(double *out, int iters, double c2d)
{
    const int lane = threadIdx.x & 63;
    double left = kBig, diag = lane == 0 ? 0.0 : kBig;
    float dc[8];
    lane_costs(dc, lane);
    const double top = 3.0 + lane;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = lane_shr1(left, top);
            double m;
            float L;
            softmin3_parts(diag, up, left, m, L);
            const double cur = fma((double)dc[u & 7], c2d, m) - (double)L;
            diag = up;
            left = cur;
        }
    }
    if (left == 12345.678) out[0] = left;
}

// Two rows per lane: lane t owns rows 2t (a) and 2t+1 (b) of a 128-row band.  At step s it computes
// the cells (2t, s-2t) and (2t+1, s-2t-1), which do not depend on each other:
//   a: up = row 2t-1 = the lane above's b of the previous step (one lane shift), diagonal = that
//      shifted value one step earlier, left = the own previous a;
//   b: up = the own a of the previous step, diagonal = the own a two steps earlier, left = own previous b.
// 128 cells per step and wavefront, one lane shift instead of two.
__global__ void dp_step_two_rows_kernel(double *out, int iters, double c2d)
{
    const int lane = threadIdx.x & 63;
    double a_left = kBig, a_diag = lane == 0 ? 0.0 : kBig, a_prev2 = kBig, b_left = kBig;
    float dc[8];
    lane_costs(dc, lane);
    const double top = 3.0 + lane;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double a_up = lane_shr1(b_left, top);
            double ma, mb;
            float La, Lb;
            softmin3_parts(a_diag, a_up, a_left, ma, La);
            softmin3_parts(a_prev2, a_left, b_left, mb, Lb);
            const double a_cur = fma((double)dc[u & 7], c2d, ma) - (double)La;
            const double b_cur = fma((double)dc[(u + 3) & 7], c2d, mb) - (double)Lb;
            a_diag = a_up;
            a_prev2 = a_left;
            a_left = a_cur;
            b_left = b_cur;
        }
    }
    if (a_left + b_left == 12345.678) out[0] = a_left;
}

// the step with the memory traffic of the real consumer added piece by piece:
//   bit 0: cost read from an LDS ring, bit 1: the value written to LDS for the neighbouring band,
//   bit 2: the value stored to a table in HBM (non-temporal, one 512-byte row per step),
//   bit 3: one workgroup barrier per 32 steps, with two more wavefronts that only take the barrier
// table: 256 workgroups x 4 macro-steps x 32 x 64 doubles, rewritten over and over.
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
    double left = kBig, diag = lane == 0 ? 0.0 : kBig;
    float dc[8];
    lane_costs(dc, lane);
    const double top = 3.0 + lane;
    const float *my_ring = ring + lane * 129;
    double *my_eo = eo + (lane == 63 ? 0 : 32 + lane);
    double *Rk = table + (size_t)blockIdx.x * 4 * 32 * 64;
    for (int it = 0; it < iters; ++it) {
        const float *rd = my_ring + (it & 3) * 32;
        double *Rs = Rk + (size_t)(it & 3) * 32 * 64;
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = lane_shr1(left, top);
            const float d = (V & 1) ? rd[u] : dc[u & 7];
            double m;
            float L;
            softmin3_parts(diag, up, left, m, L);
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
// of a workgroup (one per SIMD) run the DP step (ROWS rows per lane); wavefronts 4-7 (same SIMDs) run
// `mfma_per_iter` dependent v_mfma_f32_32x32x16_f16 per 32 steps (0: they only exist).
template <int ROWS> __global__ __launch_bounds__(512) void coexec_kernel(double *out, int iters, int mfma_per_iter, double c2d)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (w >= 4) {
        half8 a, b;
        for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(0.001f * (lane + i)); b[i] = (_Float16)(0.002f * (lane - i)); }
        floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it)
            for (int m = 0; m < mfma_per_iter; ++m) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
        if (acc[0] == 12345.678f) out[1] = acc[3];
        return;
    }
    float dc[8];
    lane_costs(dc, lane);
    const double top = 3.0 + lane;
    if (ROWS == 2) {
        double a_left = kBig, a_diag = lane == 0 ? 0.0 : kBig, a_prev2 = kBig, b_left = kBig;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const double a_up = lane_shr1(b_left, top);
                double ma, mb;
                float La, Lb;
                softmin3_parts(a_diag, a_up, a_left, ma, La);
                softmin3_parts(a_prev2, a_left, b_left, mb, Lb);
                const double a_cur = fma((double)dc[u & 7], c2d, ma) - (double)La;
                const double b_cur = fma((double)dc[(u + 3) & 7], c2d, mb) - (double)Lb;
                a_diag = a_up;
                a_prev2 = a_left;
                a_left = a_cur;
                b_left = b_cur;
            }
        }
        if (a_left + b_left == 12345.678) out[0] = a_left;
        return;
    }
    double left = kBig, diag = lane == 0 ? 0.0 : kBig;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const double up = lane_shr1(left, top);
            double m;
            float L;
            softmin3_parts(diag, up, left, m, L);
            const double cur = fma((double)dc[u & 7], c2d, m) - (double)L;
            diag = up;
            left = cur;
        }
    }
    if (left == 12345.678) out[0] = left;
}

constexpr size_t kScratchBytes = (size_t)256 * 4 * 32 * 64 * sizeof(double);  // table of dp_step_mem_kernel

// Launches one probe once.  Returns false for an unknown probe / variant.
inline bool launch(int which, int variant, int waves_per_simd, int iters, double *scratch, hipStream_t st)
{
    const int w = waves_per_simd;
    const double c2d = 14.4;
    auto rate = [&](auto op) {
        constexpr int OP = decltype(op)::value;
        if (which == 0)
            rate_kernel<OP><<<256, 256 * w, 0, st>>>(scratch, iters);
        else
            latency_kernel<OP><<<256, 256, 0, st>>>(scratch, iters);
    };
    switch (which) {
        case 0:
        case 1:
            switch (variant) {
                case ADD_F32: rate(std::integral_constant<int, ADD_F32>{}); return true;
                case FMA_F32: rate(std::integral_constant<int, FMA_F32>{}); return true;
                case ADD_F64: rate(std::integral_constant<int, ADD_F64>{}); return true;
                case MIN_F64: rate(std::integral_constant<int, MIN_F64>{}); return true;
                case FMA_F64: rate(std::integral_constant<int, FMA_F64>{}); return true;
                case EXP_F32: rate(std::integral_constant<int, EXP_F32>{}); return true;
                case LOG_F32: rate(std::integral_constant<int, LOG_F32>{}); return true;
                case CVT_F32_F64: if (which == 1) return false; rate(std::integral_constant<int, CVT_F32_F64>{}); return true;
                case CVT_F64_F32: if (which == 1) return false; rate(std::integral_constant<int, CVT_F64_F32>{}); return true;
                case MOV_DPP: rate(std::integral_constant<int, MOV_DPP>{}); return true;
                default: return false;
            }
        case 2: dp_step_kernel<<<256, 256 * w, 0, st>>>(scratch, iters, c2d); return true;
        case 3: dp_step_two_rows_kernel<<<256, 256 * w, 0, st>>>(scratch, iters, c2d); return true;
        case 4:  // variant = MFMA per 32 steps, + 1000 for two rows per lane
            if (variant >= 1000)
                coexec_kernel<2><<<256, 512, 0, st>>>(scratch, iters, variant - 1000, c2d);
            else
                coexec_kernel<1><<<256, 512, 0, st>>>(scratch, iters, variant, c2d);
            return true;
        case 5:
            switch (variant) {
                case 0: dp_step_mem_kernel<0><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 1: dp_step_mem_kernel<1><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 3: dp_step_mem_kernel<3><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 7: dp_step_mem_kernel<7><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 15: dp_step_mem_kernel<15><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 4: dp_step_mem_kernel<4><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                case 8: dp_step_mem_kernel<8><<<256, 192, 0, st>>>(scratch, iters, c2d); return true;
                default: return false;
            }
        default: return false;
    }
}

}  // namespace probe
}  // namespace sdtw
