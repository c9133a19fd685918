// Device-side building blocks: cross-lane shifts and the float32 32x32 cost block.
#pragma once
#include <hip/hip_runtime.h>

#include "layout.h"

namespace sdtw {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------------------------------------
// Cross-lane shifts over the 64 lanes of a wavefront (DPP wave_shr:1 / wave_shl:1).
// result[t] = v[t-1]; lane 0 keeps `fill`.
__device__ __forceinline__ int lane_shr1_i32(int v, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, 0x138, 0xf, 0xf, false);
}
// result[t] = v[t+1]; lane 63 keeps `fill`.
__device__ __forceinline__ int lane_shl1_i32(int v, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, 0x130, 0xf, 0xf, false);
}
// Minimum of a float over the 64 lanes (the same value in every lane's result): row-wise scan with
// row_shr 1, 2, 4, 8, then lane 15 of a row to the next row (row_bcast:15) and lane 31 to the upper
// half (row_bcast:31); lane 63 holds the minimum.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_min_step(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return fminf(v, __int_as_float(moved));
}
__device__ __forceinline__ float wave_min_f32(float v)
{
    v = dpp_min_step<0x111, 0xf>(v);
    v = dpp_min_step<0x112, 0xf>(v);
    v = dpp_min_step<0x114, 0xf>(v);
    v = dpp_min_step<0x118, 0xf>(v);
    v = dpp_min_step<0x142, 0xa>(v);
    v = dpp_min_step<0x143, 0xc>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// the same for the maximum
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_max_step(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xf, false);
    return fmaxf(v, __int_as_float(moved));
}
__device__ __forceinline__ float wave_max_f32(float v)
{
    v = dpp_max_step<0x111, 0xf>(v);
    v = dpp_max_step<0x112, 0xf>(v);
    v = dpp_max_step<0x114, 0xf>(v);
    v = dpp_max_step<0x118, 0xf>(v);
    v = dpp_max_step<0x142, 0xa>(v);
    v = dpp_max_step<0x143, 0xc>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ double lane_shr1(double v, double fill)
{
    int lo = lane_shr1_i32(__double2loint(v), __double2loint(fill));
    int hi = lane_shr1_i32(__double2hiint(v), __double2hiint(fill));
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double lane_shl1(double v, double fill)
{
    int lo = lane_shl1_i32(__double2loint(v), __double2loint(fill));
    int hi = lane_shl1_i32(__double2hiint(v), __double2hiint(fill));
    return __hiloint2double(hi, lo);
}
// value of lane `src` (compile-time constant after unrolling) broadcast to the wavefront
__device__ __forceinline__ double read_lane(double v, int src)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

// ---------------------------------------------------------------------------------------------
// One 32x32 block of inner products <x_r, y_c> on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32).  Lane l supplies row r = l&31 of both operands; lanes 0-31 and 32-63
// split every group of 8 feature indices into its lower and upper 4, so one float4 load per
// operand feeds four MFMAs.  xrow / yrow point at this lane's rows (already clamped in range).
// Result layout (hardware): acc[i] belongs to row 8*(i/4) + 4*(l>>5) + (i&3), column l&31.
__device__ __forceinline__ floatx16 dot_block_32x32(const float *__restrict__ xrow,
                                                    const float *__restrict__ yrow, int D, bool vec,
                                                    int lane)
{
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int h4 = (lane >> 5) * 4;
    if (vec) {
#pragma unroll 4
        for (int k0 = 0; k0 < D; k0 += 8) {
            const float4 a = *reinterpret_cast<const float4 *>(xrow + k0 + h4);
            const float4 b = *reinterpret_cast<const float4 *>(yrow + k0 + h4);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
    } else {
        for (int k0 = 0; k0 < D; k0 += 8) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int k = k0 + h4 + c;
                const float a = (k < D) ? xrow[k] : 0.f;
                const float b = (k < D) ? yrow[k] : 0.f;
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
            }
        }
    }
    return acc;
}

__device__ __forceinline__ int acc_row(int i, int lane) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }

// Squared-Euclidean cost block through the norm expansion (Sec. 4.3, Eq. 8):
//   d = ||x_i||^2 - 2 <x_i,y_j> + ||y_j||^2, clamped at 0 (rounding can push it below).
// Rows i0.., columns j0.. of pair data (xb, yb, xnb, ynb); rows/columns outside the grid are
// computed from clamped indices and must be ignored by the caller.
__device__ __forceinline__ void cost_block(const Params &p, const float *__restrict__ xb,
                                           const float *__restrict__ yb,
                                           const float *__restrict__ xnb,
                                           const float *__restrict__ ynb, int i0, int j0, int lane,
                                           float (&out)[16])
{
    const int r = lane & 31;
    const int xi = min(i0 + r, p.N - 1), yj = min(j0 + r, p.M - 1);
    const floatx16 acc = dot_block_32x32(xb + (size_t)xi * p.D, yb + (size_t)yj * p.D, p.D,
                                         p.vec_xy != 0, lane);
    const float ynv = ynb[yj];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = min(i0 + acc_row(i, lane), p.N - 1);
        out[i] = fmaxf(xnb[row] + ynv - 2.0f * acc[i], 0.0f);
    }
}

// Length of pair b's sequence when the batch is ragged (lens != nullptr), clamped to [1, full].
__device__ __forceinline__ int pair_len(const int32_t *lens, int b, int full)
{
    if (lens == nullptr) return full;
    return __builtin_amdgcn_readfirstlane(max(1, min(lens[b], full)));
}

// Macro-steps a band sweep has to run when only cells with |i-j| <= window belong to the grid.
// The band(s) cover rows [row_a, row_b + 63] (row_a == row_b for one band; a chained pair runs the
// union).  Lane t meets column j at step j + t, so the cells inside the window lie at steps
// [row_a - w, row_b + 126 + w]; one more step on either side keeps every predecessor that a cell
// inside the window reads - itself outside the window - among the computed cells (cost kBigCost)
// or the initial state (kBig).  Macro-steps [lo, hi] are run; hi_u is hi before it is clipped to
// the table: a 32x32 block (rb, cb) of the band holds cells of macro-steps cb+rb and cb+rb+1 and is
// either complete within [lo, hi_u] or entirely outside the window.
//
// Ragged batches: with Nl, Ml the lengths of the pair (the largest ones among the pairs a workgroup
// serves) the sweep also stops after the macro-step (Ml+63)/32, which still holds every cell of the
// column blocks 0 .. cb_last = (Ml-1)/32, and bands that start at or below row Nl do not run at all
// (hi < lo).  Nl = N, Ml = M change nothing.
struct SweepRange { int lo, hi, hi_u, cb_last; };

__device__ __forceinline__ SweepRange sweep_range(const Params &p, int row_a, int row_b, int Nl, int Ml)
{
    SweepRange r;
    r.cb_last = (Ml - 1) / kBlk;
    if (p.window >= kNoWindow) {
        r.lo = 0;
        r.hi = p.nmacro - 1;
        r.hi_u = kNoWindow;
    } else {
        const int first = row_a - p.window - 1;
        r.lo = first > 0 ? first / kBlk : 0;
        r.hi_u = (row_b + 2 * kBandRows - 1 + p.window) / kBlk;
        r.hi = min(r.hi_u, p.nmacro - 1);
        r.lo = min(r.lo, r.hi);
    }
    if (Ml < p.M) r.hi = min(r.hi, (Ml + 2 * kBlk - 1) / kBlk);
    if (row_a >= Nl) {
        r.lo = 0;
        r.hi = -1;
        r.hi_u = -1;
    }
    return r;
}

__device__ __forceinline__ SweepRange sweep_range(const Params &p, int row_a, int row_b)
{
    return sweep_range(p, row_a, row_b, p.N, p.M);
}

// pair_len without the promise that all lanes ask for the same pair
__device__ __forceinline__ int pair_len_lane(const int32_t *lens, int b, int full)
{
    return lens == nullptr ? full : max(1, min(lens[b], full));
}

// First macro-step held by the tables (R, Q, checkpoints) of band k: that of the widest range the
// band may run, alone or in a chained pair with the band above it.
__device__ __forceinline__ int table_base(const Params &p, int k)
{
    if (p.window >= kNoWindow) return 0;
    const int r = max(k - 1, 0) * kBandRows;
    return sweep_range(p, r, r).lo;
}

__device__ __forceinline__ bool in_window(int i, int j, int w)
{
    return (unsigned)(j - i + w) <= 2u * (unsigned)w;
}

}  // namespace sdtw
