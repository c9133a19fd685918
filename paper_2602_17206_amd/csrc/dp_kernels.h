// Forward and backward DP kernels (the dependent anti-diagonal sweeps) for gfx950.
//
// Geometry.  A band is 64 consecutive rows of one pair; one wavefront owns it, lane t owning row
// row0+t.  At step s lane t is at column j = s - t, so the 64 cells of a step lie on one
// anti-diagonal and are independent (Sec. 4.1).  A cell's three neighbours are the lane's own
// previous value, the adjacent lane's previous value (one DPP wave shift) and that same value one
// step earlier, so the dependent chain never leaves the registers.  Steps come in macro-steps of 32.
//
// Cells outside the N x M grid are not masked.  They are fed a huge finite cost (kBigCost) and the
// table boundary is a huge finite value (kBig) instead of +inf: a cell whose three neighbours are
// all kBig stays exactly kBig (kBig + kBigCost == kBig in float64), a grid cell sees
// (float)(kBig - m) = +inf and 2^-inf = 0 for such a neighbour, exactly as Sec. 2's boundary
// conditions R[i,0] = R[0,j] = +inf demand, and no inf - inf = NaN can arise.  Cells right of
// column M or below row N get finite garbage that no grid cell depends on.
//
// Cost values reach the lanes through an LDS ring indexed by STEP, not by column:
// cell (band row t, column j) lives at ring[t][(j + t) mod 96].  At step s every lane reads
// position s mod 96 of its own row, so the address of a step is a per-macro-step base plus an
// immediate, and three phases of 32 steps are live at any time: the one being read and the two
// being filled for later.  32x32 cost blocks are written into the ring with that skew applied.
#pragma once
#include <hip/hip_runtime.h>

#include "device_core.h"
#include "layout.h"

namespace sdtw {

constexpr int kRingCols = 96;     // three phases of 32 steps
constexpr int kRingStride = 97;   // floats per band row in LDS (odd: lanes hit distinct banks)
constexpr double kBig = 1e300;    // stands for +inf in the DP tables
constexpr float kBigCost = 3.0e38f;  // cost of a cell outside the grid
constexpr int kStatusTimeoutDp = 6;  // SDTW_ERR_TIMEOUT

__device__ __forceinline__ double min_f64(double a, double b)
{
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// softmin_gamma(a,b,c) split as  m - corr  with  m = min(a,b,c) (float64) and
// corr = gamma ln(sum_k exp(-(v_k - m)/gamma)) (float32, >= 0).   (Sec. 2 Eq. 2; max-shift of Sec. 4.2)
__device__ __forceinline__ void softmin3_parts(double a, double b, double c, float c2, float gamma_ln2,
                                               double &m, float &corr)
{
    m = min_f64(min_f64(a, b), c);
    const float fa = (float)(a - m), fb = (float)(b - m), fc = (float)(c - m);
    const float mx = __builtin_fmaxf(__builtin_fmaxf(fa, fb), fc);
    const float md = __builtin_amdgcn_fmed3f(fa, fb, fc);
    const float S = 1.0f + __builtin_amdgcn_exp2f(-md * c2) + __builtin_amdgcn_exp2f(-mx * c2);
    corr = gamma_ln2 * __builtin_amdgcn_logf(S);
}

__device__ __forceinline__ float comp4(const float4 &v, int c)
{
    return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

// MFMA operand of one 32-row block: lane (r = lane&31, h = lane>>5) keeps, for every group of 8
// features, the 4 features 8c+4h .. 8c+4h+3 of row r.  Features >= D are zero.
template <int KCH>
__device__ __forceinline__ void load_operand(float4 (&dst)[KCH], const float *__restrict__ rowptr, int D,
                                             int h4, bool vec, float scale)
{
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
        const int k = 8 * c + h4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vec) {
            if (k < D) v = *reinterpret_cast<const float4 *>(rowptr + k);
        } else {
            if (k + 0 < D) v.x = rowptr[k + 0];
            if (k + 1 < D) v.y = rowptr[k + 1];
            if (k + 2 < D) v.z = rowptr[k + 2];
            if (k + 3 < D) v.w = rowptr[k + 3];
        }
        dst[c] = make_float4(v.x * scale, v.y * scale, v.z * scale, v.w * scale);
    }
}

// One whole 32x32 cost block from register operands:  sum_k (-2 x_ik) y_jk + ||x_i||^2 * 1 + 1 * ||y_j||^2
// (Sec. 4.3 Eq. 8 with the two norm terms fed through one extra MFMA).
template <int KCH>
__device__ __forceinline__ floatx16 block_from_regs(const float4 (&xa)[KCH], float ax, const float4 (&yb)[KCH],
                                                    float by)
{
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < KCH; ++c) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[c].x, yb[c].x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[c].y, yb[c].y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[c].z, yb[c].z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[c].w, yb[c].w, acc, 0, 0, 0);
    }
    return __builtin_amdgcn_mfma_f32_32x32x2f32(ax, by, acc, 0, 0, 0);
}

// Writes a 32x32 cost block given in MFMA accumulator layout into the step-indexed ring.
// Block rows are band rows 32*rb .., columns 32*cb ..; entries outside the grid become kBigCost.
__device__ __forceinline__ void store_block_acc(float *ring, const floatx16 &acc, int rb, int cb, int row0, int N,
                                                int M, int lane)
{
    const int h = lane >> 5, c = lane & 31;
    int ph = (cb + rb) % 3;
    if (ph < 0) ph += 3;
    const unsigned sbase = (unsigned)ph * 32u + (unsigned)(c + 4 * h);
    float *rowbase = ring + (32 * rb + 4 * h) * kRingStride;
    const int i0 = row0 + 32 * rb, j0 = 32 * cb;
    const bool inside = (i0 + 32 <= N) && (j0 >= 0) && (j0 + 32 <= M);
    const bool col_ok = (unsigned)(j0 + c) < (unsigned)M;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int rr = 8 * (i >> 2) + (i & 3);  // + 4h = row inside the block
        unsigned pos = sbase + (unsigned)rr;
        pos = min(pos, pos - (unsigned)kRingCols);
        float v = fmaxf(acc[i], 0.0f);
        if (!inside) v = (col_ok && (i0 + 4 * h + rr < N)) ? v : kBigCost;
        rowbase[rr * kRingStride + pos] = v;
    }
}

// Unfused mode: the 32x32 block of the stored cost tensor as 4 float4 per lane
// (lane -> row (lane>>3) + 8*it of the block, columns 4*(lane&7) ..), kBigCost outside the grid.
__device__ __forceinline__ void load_cost_block(float4 (&v)[4], const float *__restrict__ cost_b, int rb, int cb,
                                                int row0, int N, int M, bool vec_m, int lane)
{
    const int c4 = (lane & 7) * 4, j0 = 32 * cb;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = row0 + 32 * rb + (lane >> 3) + 8 * it;
        const int col = j0 + c4;
        float4 t = make_float4(kBigCost, kBigCost, kBigCost, kBigCost);
        if (row < N && col >= 0) {
            const float *q = cost_b + (size_t)row * M + col;
            if (vec_m && col + 3 < M) {
                t = *reinterpret_cast<const float4 *>(q);
            } else {
                if (col + 0 < M) t.x = q[0];
                if (col + 1 < M) t.y = q[1];
                if (col + 2 < M) t.z = q[2];
                if (col + 3 < M) t.w = q[3];
            }
        }
        v[it] = t;
    }
}

__device__ __forceinline__ void store_cost_block(float *ring, const float4 (&v)[4], int rb, int cb, int lane)
{
    int ph = (cb + rb) % 3;
    if (ph < 0) ph += 3;
    const int c4 = (lane & 7) * 4;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = (lane >> 3) + 8 * it;
        float *rowp = ring + (32 * rb + r) * kRingStride;
        const unsigned base = (unsigned)ph * 32u + (unsigned)(c4 + r);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsigned pos = base + (unsigned)e;
            pos = min(pos, pos - (unsigned)kRingCols);
            rowp[pos] = comp4(v[it], e);
        }
    }
}

// Boundary values travel between bands through a buffer pre-filled with kSentinel; each value is
// published with one 64-bit device-scope atomic store, so it validates itself (no flag, no fence).
// `bits` holds what an earlier prefetch saw.  Polls until all needed lanes have a value; a band
// gives up after p.spin_limit polls, records SDTW_ERR_TIMEOUT and never waits again; other bands
// notice the recorded status and stop waiting too, so every kernel exits.
__device__ __forceinline__ double resolve_boundary(const Params &p, const unsigned long long *row, int jj, bool need,
                                                   int lane, bool &gave_up, unsigned long long bits)
{
    unsigned spins = 0;
    for (;;) {
        const bool ok = !need || bits != kSentinel;
        if (__all(ok) || gave_up) break;
        ++spins;
        bool stop = spins > p.spin_limit;
        if (!stop && (spins & 255u) == 0)
            stop = __hip_atomic_load(&p.hdr->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == kStatusTimeoutDp;
        if (stop) {
            if (lane == 0) atomicMax(&p.hdr->status, kStatusTimeoutDp);
            gave_up = true;
            break;
        }
        __builtin_amdgcn_s_sleep(4);
        if (need) bits = __hip_atomic_load(row + jj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return __longlong_as_double((long long)bits);
}

__device__ __forceinline__ unsigned long long peek_boundary(const unsigned long long *row, int jj, bool need)
{
    unsigned long long bits = (unsigned long long)__double_as_longlong(kBig);
    if (need) bits = __hip_atomic_load(row + jj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return bits;
}

__device__ __forceinline__ void publish_boundary(unsigned long long *row, int j, double v)
{
    __hip_atomic_store(row + j, (unsigned long long)__double_as_longlong(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// How the cost blocks are made.
//   KCH > 0 : fused, D <= 8*KCH: operands live in registers, MFMAs are interleaved with the DP steps
//   KCH == 0: fused, any D: blocks are computed between macro-steps straight from x and y
//   KCH < 0 : unfused: blocks are loaded from the stored cost tensor one macro-step ahead
template <int KCH> struct CostRegs {
    float4 xa[2][KCH > 0 ? KCH : 1];  // -2 * x rows of the two 32-row blocks
    float ax[2];                      // lanes 0-31: ||x_r||^2, lanes 32-63: 1
    float4 ya[KCH > 0 ? KCH : 1];     // y rows of the newer column block
    float4 yb[KCH > 0 ? KCH : 1];     // y rows of the older column block
    float bya, byb;                   // lanes 0-31: 1, lanes 32-63: ||y_c||^2
};

template <int KCH>
__device__ __forceinline__ void load_y_block(const Params &p, const float *yb_ptr, const float *ynb, int cb, int lane,
                                             float4 (&dst)[KCH > 0 ? KCH : 1], float &by)
{
    if constexpr (KCH > 0) {
        int col = 32 * cb + (lane & 31);
        col = max(0, min(col, p.M - 1));
        load_operand<KCH>(dst, yb_ptr + (size_t)col * p.D, p.D, (lane >> 5) * 4, p.vec_d4 != 0, 1.0f);
        by = (lane >> 5) ? ynb[col] : 1.0f;
    }
}

// Generic-D cost block between macro-steps (no register operands).
__device__ __forceinline__ void sync_block_generic(const Params &p, int b, float *ring, int rb, int cb, int row0,
                                                   int lane)
{
    float out[16];
    const int i0 = row0 + 32 * rb, j0 = 32 * cb;
    cost_block(p, p.x + b * p.x_stride, p.y + b * p.y_stride, p.xn + b * p.xn_stride, p.yn + b * p.yn_stride,
               min(i0, p.N - 1), max(0, min(j0, p.M - 1)), lane, out);
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = out[i];
    // cost_block clamps row/column indices itself; entries outside the grid are replaced on store.
    // When the block origin had to be clamped the whole block is outside the grid.
    const bool origin_ok = (i0 < p.N) && (j0 >= 0) && (j0 < p.M);
    store_block_acc(ring, acc, rb, cb, row0, origin_ok ? p.N : 0, p.M, lane);
}

// ---------------------------------------------------------------------------------------------
// Forward DP (Sec. 2 Eq. 1-2 in the anti-diagonal order of Sec. 4.1).
// Band tasks are handed out by an atomic ticket in band-major order: a band only ever waits for a
// band with a smaller ticket, which is running or done, so the wait ends whatever order the
// hardware starts workgroups in.  The table goes to HBM step-major, R[b][band][s][lane]: one
// coalesced 512-byte store per step; the band's last row goes to the boundary buffer.
// ---------------------------------------------------------------------------------------------
template <int KCH>
__global__ __launch_bounds__(64) void forward_dp_kernel(Params p, float *__restrict__ value)
{
    __shared__ float ring[kBandRows * kRingStride];
    constexpr bool FUSED_REG = KCH > 0;
    constexpr bool UNFUSED = KCH < 0;
    constexpr int KR = KCH > 0 ? KCH : 1;

    const int lane = threadIdx.x;
    unsigned ticket = 0;
    if (lane == 0) ticket = atomicAdd(&p.hdr->fwd_ticket, 1u);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    const int k = ticket / (unsigned)p.B;
    const int b = ticket - k * p.B;
    if (k >= p.nbands) return;

    const int M = p.M, N = p.N;
    const int row0 = k * kBandRows;
    const float c2 = p.inv_gamma_log2e, g2 = p.gamma_ln2;
    const float *xb = p.x + b * p.x_stride, *yb_ptr = p.y + b * p.y_stride;
    const float *xnb = p.xn + b * p.xn_stride, *ynb = p.yn + b * p.yn_stride;
    const float *cost_b = UNFUSED ? p.cost + (size_t)b * N * M : nullptr;

    for (int e = lane; e < kBandRows * kRingStride; e += 64) ring[e] = kBigCost;

    CostRegs<KCH> cr;
    if constexpr (FUSED_REG) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int row = min(row0 + 32 * rb + (lane & 31), N - 1);
            load_operand<KR>(cr.xa[rb], xb + (size_t)row * p.D, p.D, (lane >> 5) * 4, p.vec_d4 != 0, -2.0f);
            cr.ax[rb] = (lane >> 5) ? 1.0f : xnb[row];
        }
    }
    __syncthreads();

    // cost block (upper rows, column block 0) is needed by the very first macro-step
    float4 pre[2][4];
    if constexpr (FUSED_REG) {
        load_y_block<KCH>(p, yb_ptr, ynb, 0, lane, cr.yb, cr.byb);
        const floatx16 acc = block_from_regs<KR>(cr.xa[0], cr.ax[0], cr.yb, cr.byb);
        store_block_acc(ring, acc, 0, 0, row0, N, M, lane);
    } else if constexpr (UNFUSED) {
        load_cost_block(pre[0], cost_b, 0, 0, row0, N, M, p.vec_m != 0, lane);
        store_cost_block(ring, pre[0], 0, 0, lane);
    } else {
        sync_block_generic(p, b, ring, 0, 0, row0, lane);
    }

    bool gave_up = false;
    double left = kBig;                                  // R[i][j-1]
    double diag = (k == 0 && lane == 0) ? 0.0 : kBig;    // R[i-1][j-1]; R[0,0] = 0 in the paper's indexing
    double edge = kBig;                                  // collects lane 63's values of a macro-step
    const unsigned long long *brow_in = p.brow + ((size_t)b * p.nbands + (k > 0 ? k - 1 : 0)) * M;
    unsigned long long *brow_out = p.brow + ((size_t)b * p.nbands + k) * M;
    double *Rw = p.R + ((size_t)b * p.nbands + k) * (size_t)p.nmacro * kBlk * kBandRows + lane;
    const bool emit_bottom = (k + 1 < p.nbands);
    const float *my_ring = ring + lane * kRingStride;

    // row above the band for macro-step 0: lane l < 32 holds column l
    double topv = kBig;
    if (k > 0) {
        const bool need = lane < kBlk && lane < M;
        topv = resolve_boundary(p, brow_in, lane, need, lane, gave_up, peek_boundary(brow_in, lane, need));
    }
    __syncthreads();

    for (int sg = 0; sg < p.nmacro; ++sg) {
        // ---- prefetches for the next macro-step
        unsigned long long nxt_bits = (unsigned long long)__double_as_longlong(kBig);
        const int jn = (sg + 1) * kBlk + lane;
        const bool need_n = (k > 0) && lane < kBlk && jn < M;
        if (k > 0) nxt_bits = peek_boundary(brow_in, jn, need_n);
        floatx16 acc0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        floatx16 acc1 = acc0;
        if constexpr (FUSED_REG) load_y_block<KCH>(p, yb_ptr, ynb, sg + 1, lane, cr.ya, cr.bya);
        if constexpr (UNFUSED) {
            load_cost_block(pre[0], cost_b, 1, sg, row0, N, M, p.vec_m != 0, lane);
            load_cost_block(pre[1], cost_b, 0, sg + 1, row0, N, M, p.vec_m != 0, lane);
        }
        const float *rd = my_ring + (sg % 3) * kBlk;
        double *Rs = Rw + (size_t)sg * kBlk * kBandRows;

        // ---- 32 steps; the MFMAs of the two blocks the NEXT macro-step needs are spread over them:
        //      first half: (lower rows, column block sg) with y block sg; second half: (upper rows, sg+1)
#pragma unroll
        for (int u = 0; u < kBlk; ++u) {
            const double up = lane_shr1(left, topv);  // R[i-1][j]; lane 0 takes the row above the band
            topv = lane_shl1(topv, topv);
            const float dc = rd[u];
            double m;
            float corr;
            softmin3_parts(diag, up, left, c2, g2, m, corr);
            // all additions that build the table are float64: a float32 rounding of d - corr here
            // would differ between the two sweeps and add up along the alignment path
            const double cur = (m - (double)corr) + (double)dc;
            Rs[u * kBandRows] = cur;
            edge = lane_shl1(edge, cur);  // lane 63 keeps its own value, the others move down
            diag = up;
            left = cur;
            if constexpr (FUSED_REG) {
#pragma unroll
                for (int mi = u * KR / 4; mi < (u + 1) * KR / 4; ++mi) {
                    const int blk = mi / (4 * KR), c = (mi % (4 * KR)) / 4, e = mi % 4;
                    if (blk == 0)
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(comp4(cr.xa[1][c], e), comp4(cr.yb[c], e), acc0, 0, 0, 0);
                    else
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(comp4(cr.xa[0][c], e), comp4(cr.ya[c], e), acc1, 0, 0, 0);
                }
                if (u == 15) acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cr.ax[1], cr.byb, acc0, 0, 0, 0);
                if (u == 31) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cr.ax[0], cr.bya, acc1, 0, 0, 0);
            }
        }

        // ---- last row of the band: lanes 32..63 hold columns 32*sg - 63 + (lane - 32)
        if (emit_bottom && lane >= kBlk) {
            const int j = sg * kBlk + lane - kBlk - (kBandRows - 1);
            if (j >= 0 && j < M) publish_boundary(brow_out, j, edge);
        }
        // ---- cost blocks for the next macro-step
        if constexpr (FUSED_REG) {
            store_block_acc(ring, acc0, 1, sg, row0, N, M, lane);
            store_block_acc(ring, acc1, 0, sg + 1, row0, N, M, lane);
#pragma unroll
            for (int c = 0; c < KR; ++c) cr.yb[c] = cr.ya[c];
            cr.byb = cr.bya;
        } else if constexpr (UNFUSED) {
            store_cost_block(ring, pre[0], 1, sg, lane);
            store_cost_block(ring, pre[1], 0, sg + 1, lane);
        } else {
            sync_block_generic(p, b, ring, 1, sg, row0, lane);
            sync_block_generic(p, b, ring, 0, sg + 1, row0, lane);
        }
        // ---- row above the band for the next macro-step
        if (k > 0) topv = resolve_boundary(p, brow_in, jn, need_n, lane, gave_up, nxt_bits);
        __syncthreads();
    }

    // R[N,M] of the pair: cell (N-1, M-1) was stored at step M-1+lane by the lane that owns row N-1
    if (row0 + lane == N - 1) {
        const double r = Rw[(size_t)(M - 1 + lane) * kBandRows];
        p.rfinal[b] = r;
        value[b] = (float)r;
    }
}

// ---------------------------------------------------------------------------------------------
// Backward DP (Sec. 2 "Backward pass", Sec. 4.2).
//
// The paper carries Ebar = log E with
//   Ebar[i,j] = logsumexp(Ebar[i+1,j]+alpha, Ebar[i,j+1]+beta, Ebar[i+1,j+1]+delta),
//   alpha = (R[i+1,j] - R[i,j] - d[i+1,j])/gamma  (beta, delta alike).
// Substituting T[i,j] := R[N,M] - gamma*Ebar[i,j] - R[i,j] + d[i,j] turns this, term by term, into
//   T[i,j] = d[i,j] + softmin_gamma(T[i+1,j], T[i,j+1], T[i+1,j+1]),   T[N+1,M+1] := 0,
//   Ebar[i,j] = (R[N,M] - R[i,j] - (T[i,j] - d[i,j])) / gamma,
// the same log-space recurrence with the logarithm scaled by gamma.  It is still max-shifted
// log-sum-exp arithmetic (nothing can overflow for small gamma), it needs one cost value per cell
// instead of three, and the only subtraction of large numbers, R[N,M] - R[i,j] - m, happens once per
// cell in float64.  E = exp(Ebar) is applied per cell as soon as Ebar is known.
//
// Bands run bottom-up; lane t needs lane t+1's values, the band below supplies lane 63's.
// E replaces the consumed cost value in the ring and leaves as row-major 32x32 blocks, with one
// flag byte per block saying whether any entry is non-zero.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void flush_E_block(const Params &p, const float *ring, float *__restrict__ Eb,
                                              unsigned char *__restrict__ nzb, int rb, int cb, int row0, int lane)
{
    if (cb < 0 || cb >= p.ncb || row0 + 32 * rb >= p.N) return;
    int ph = (cb + rb) % 3;
    if (ph < 0) ph += 3;
    const int c4 = (lane & 7) * 4, j0 = cb * kBlk;
    bool any = false;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = (lane >> 3) + 8 * it;
        const int row = row0 + rb * 32 + r;
        const float *rowp = ring + (32 * rb + r) * kRingStride;
        const unsigned base = (unsigned)ph * 32u + (unsigned)(c4 + r);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsigned pos = base + (unsigned)e;
            pos = min(pos, pos - (unsigned)kRingCols);
            v[e] = rowp[pos];
        }
        if (row < p.N) {
            float *q = Eb + (size_t)row * p.M + j0 + c4;
            if (p.vec_m && j0 + c4 + 3 < p.M) {
                *reinterpret_cast<float4 *>(q) = make_float4(v[0], v[1], v[2], v[3]);
                any |= (v[0] != 0.f) | (v[1] != 0.f) | (v[2] != 0.f) | (v[3] != 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j0 + c4 + e < p.M) { q[e] = v[e]; any |= v[e] != 0.f; }
            }
        }
    }
    const bool blk_any = __any(any);
    if (lane == 0) nzb[(size_t)(row0 / kBlk + rb) * p.ncb + cb] = blk_any ? 1 : 0;
}

template <int KCH>
__global__ __launch_bounds__(64) void backward_dp_kernel(Params p)
{
    __shared__ float ring[kBandRows * kRingStride];
    constexpr bool FUSED_REG = KCH > 0;
    constexpr bool UNFUSED = KCH < 0;
    constexpr int KR = KCH > 0 ? KCH : 1;

    const int lane = threadIdx.x;
    if (p.hdr->abort_backward) return;
    unsigned ticket = 0;
    if (lane == 0) ticket = atomicAdd(&p.hdr->bwd_ticket, 1u);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    const int kk = ticket / (unsigned)p.B;
    const int b = ticket - kk * p.B;
    if (kk >= p.nbands) return;
    const int k = p.nbands - 1 - kk;

    const int M = p.M, N = p.N;
    const int row0 = k * kBandRows;
    const float c2 = p.inv_gamma_log2e, g2 = p.gamma_ln2;
    const float *xb = p.x + b * p.x_stride, *yb_ptr = p.y + b * p.y_stride;
    const float *xnb = p.xn + b * p.xn_stride, *ynb = p.yn + b * p.yn_stride;
    const float *cost_b = UNFUSED ? p.cost + (size_t)b * N * M : nullptr;
    float *Eb = p.E + (size_t)b * N * M;
    unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;

    for (int e = lane; e < kBandRows * kRingStride; e += 64) ring[e] = kBigCost;

    CostRegs<KCH> cr;
    if constexpr (FUSED_REG) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int row = min(row0 + 32 * rb + (lane & 31), N - 1);
            load_operand<KR>(cr.xa[rb], xb + (size_t)row * p.D, p.D, (lane >> 5) * 4, p.vec_d4 != 0, -2.0f);
            cr.ax[rb] = (lane >> 5) ? 1.0f : xnb[row];
        }
    }
    __syncthreads();

    // blocks the first macro-step reads: (upper rows, sg0-1), (lower rows, sg0-2) and (lower rows, sg0-1)
    const int sg0 = p.nmacro - 1;
    float4 pre[2][4];
    if constexpr (FUSED_REG) {
        load_y_block<KCH>(p, yb_ptr, ynb, sg0 - 1, lane, cr.ya, cr.bya);
        floatx16 acc = block_from_regs<KR>(cr.xa[0], cr.ax[0], cr.ya, cr.bya);
        store_block_acc(ring, acc, 0, sg0 - 1, row0, N, M, lane);
        acc = block_from_regs<KR>(cr.xa[1], cr.ax[1], cr.ya, cr.bya);
        store_block_acc(ring, acc, 1, sg0 - 1, row0, N, M, lane);
        load_y_block<KCH>(p, yb_ptr, ynb, sg0 - 2, lane, cr.yb, cr.byb);
        acc = block_from_regs<KR>(cr.xa[1], cr.ax[1], cr.yb, cr.byb);
        store_block_acc(ring, acc, 1, sg0 - 2, row0, N, M, lane);
    } else if constexpr (UNFUSED) {
        load_cost_block(pre[0], cost_b, 0, sg0 - 1, row0, N, M, p.vec_m != 0, lane);
        store_cost_block(ring, pre[0], 0, sg0 - 1, lane);
        load_cost_block(pre[0], cost_b, 1, sg0 - 1, row0, N, M, p.vec_m != 0, lane);
        store_cost_block(ring, pre[0], 1, sg0 - 1, lane);
        load_cost_block(pre[0], cost_b, 1, sg0 - 2, row0, N, M, p.vec_m != 0, lane);
        store_cost_block(ring, pre[0], 1, sg0 - 2, lane);
    } else {
        sync_block_generic(p, b, ring, 0, sg0 - 1, row0, lane);
        sync_block_generic(p, b, ring, 1, sg0 - 1, row0, lane);
        sync_block_generic(p, b, ring, 1, sg0 - 2, row0, lane);
    }

    bool gave_up = false;
    double right = kBig;  // T[i][j+1]
    double diag = kBig;   // T[i+1][j+1]
    double edge = kBig;   // collects lane 0's values of a macro-step
    // step at which this lane meets the cell whose diagonal successor is T[N+1,M+1] = 0
    const int s_corner = (row0 + lane == N - 1) ? (M - 1 + lane) : -1;
    const double Rfin = p.rfinal[b];
    const bool has_below = (k + 1 < p.nbands);
    const unsigned long long *brow_in = p.brow + ((size_t)b * p.nbands + (has_below ? k + 1 : k)) * M;
    unsigned long long *brow_out = p.brow + ((size_t)b * p.nbands + k) * M;
    const double *Rw = p.R + ((size_t)b * p.nbands + k) * (size_t)p.nmacro * kBlk * kBandRows + lane;
    float *my_ring = ring + lane * kRingStride;

    // R of the first macro-step; afterwards each value is reloaded one macro-step ahead, right after use
    double Rq[kBlk];
#pragma unroll
    for (int u = 0; u < kBlk; ++u) Rq[u] = Rfin - Rw[((size_t)sg0 * kBlk + u) * kBandRows];

    // row below the band for the first macro-step: lane l >= 32 holds column 32*sg - 63 + (l - 32)
    double botv = kBig;
    if (has_below) {
        const int jj = sg0 * kBlk + lane - kBlk - (kBandRows - 1);
        const bool need = lane >= kBlk && jj >= 0 && jj < M;
        botv = resolve_boundary(p, brow_in, jj, need, lane, gave_up, peek_boundary(brow_in, jj, need));
    }
    __syncthreads();

    for (int sg = sg0; sg >= 0; --sg) {
        unsigned long long nxt_bits = (unsigned long long)__double_as_longlong(kBig);
        const int jn = (sg - 1) * kBlk + lane - kBlk - (kBandRows - 1);
        const bool need_n = has_below && lane >= kBlk && jn >= 0 && jn < M;
        if (has_below) nxt_bits = peek_boundary(brow_in, jn, need_n);
        floatx16 acc0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        floatx16 acc1 = acc0;
        // this macro-step prepares (upper rows, sg-2) with y block sg-2 (held) and (lower rows, sg-3) with y block sg-3 (new)
        if constexpr (FUSED_REG) {
#pragma unroll
            for (int c = 0; c < KR; ++c) cr.yb[c] = cr.ya[c];
            cr.byb = cr.bya;
            if (sg == sg0) load_y_block<KCH>(p, yb_ptr, ynb, sg - 2, lane, cr.yb, cr.byb);
            load_y_block<KCH>(p, yb_ptr, ynb, sg - 3, lane, cr.ya, cr.bya);
        }
        if constexpr (UNFUSED) {
            load_cost_block(pre[0], cost_b, 0, sg - 2, row0, N, M, p.vec_m != 0, lane);
            load_cost_block(pre[1], cost_b, 1, sg - 3, row0, N, M, p.vec_m != 0, lane);
        }
        float *rd = my_ring + (sg % 3) * kBlk;
        const double *Rn = Rw + (size_t)(sg > 0 ? sg - 1 : 0) * kBlk * kBandRows;
        const int sbase = sg * kBlk;

#pragma unroll
        for (int u = kBlk - 1; u >= 0; --u) {
            const double down = lane_shl1(right, botv);  // T[i+1][j]; lane 63 takes the row below the band
            botv = lane_shr1(botv, botv);
            const float dc = rd[u];
            const double dg = (sbase + u == s_corner) ? 0.0 : diag;
            double m;
            float corr;
            softmin3_parts(dg, down, right, c2, g2, m, corr);
            const double cur = (m - (double)corr) + (double)dc;
            // gamma*Ebar = R[N,M] - R[i,j] - (m - corr)
            const float gE = (float)(Rq[u] - m) + corr;
            rd[u] = __builtin_amdgcn_exp2f(gE * c2);
            Rq[u] = Rfin - Rn[u * kBandRows];
            edge = lane_shr1(edge, cur);  // lane 0 keeps its own value, the others move up
            diag = down;
            right = cur;
            if constexpr (FUSED_REG) {
                const int v = kBlk - 1 - u;
#pragma unroll
                for (int mi = v * KR / 4; mi < (v + 1) * KR / 4; ++mi) {
                    const int blk = mi / (4 * KR), c = (mi % (4 * KR)) / 4, e = mi % 4;
                    if (blk == 0)
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(comp4(cr.xa[0][c], e), comp4(cr.yb[c], e), acc0, 0, 0, 0);
                    else
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(comp4(cr.xa[1][c], e), comp4(cr.ya[c], e), acc1, 0, 0, 0);
                }
                if (v == 15) acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cr.ax[0], cr.byb, acc0, 0, 0, 0);
                if (v == 31) acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cr.ax[1], cr.bya, acc1, 0, 0, 0);
            }
        }
        __syncthreads();

        // first row of the band, columns 32*sg .. 32*sg+31, for the band above
        if (k > 0 && lane < kBlk) {
            const int j = sg * kBlk + lane;
            if (j < M) publish_boundary(brow_out, j, edge);
        }
        // E blocks completed by this macro-step: (upper rows, sg) and (lower rows, sg-1)
        flush_E_block(p, ring, Eb, nzb, 0, sg, row0, lane);
        flush_E_block(p, ring, Eb, nzb, 1, sg - 1, row0, lane);
        __syncthreads();
        // cost blocks for the next macro-step
        if constexpr (FUSED_REG) {
            store_block_acc(ring, acc0, 0, sg - 2, row0, N, M, lane);
            store_block_acc(ring, acc1, 1, sg - 3, row0, N, M, lane);
        } else if constexpr (UNFUSED) {
            store_cost_block(ring, pre[0], 0, sg - 2, lane);
            store_cost_block(ring, pre[1], 1, sg - 3, lane);
        } else {
            sync_block_generic(p, b, ring, 0, sg - 2, row0, lane);
            sync_block_generic(p, b, ring, 1, sg - 3, row0, lane);
        }
        if (has_below) botv = resolve_boundary(p, brow_in, jn, need_n, lane, gave_up, nxt_bits);
        __syncthreads();
    }
}

}  // namespace sdtw
