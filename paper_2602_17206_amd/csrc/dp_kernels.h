// Forward and backward DP kernels (the dependent anti-diagonal sweeps) for gfx950.
//
// Geometry.  A band is 64 consecutive rows of one pair; one wavefront (the band's CONSUMER) owns
// it, lane t owning row row0+t.  At step s lane t is at column j = s - t, so the 64 cells of a step
// lie on one anti-diagonal and are independent (Sec. 4.1).  A cell's three neighbours are the
// lane's own previous value, the adjacent lane's previous value (one DPP wave shift) and that same
// value one step earlier, so the dependent chain never leaves the registers.  Steps come in
// macro-steps of 32.
//
// Workgroup (large problems).  4 bands (the same band index of 4 consecutive pairs): per band one
// consumer (the DP chain, pure VALU) and one or two PRODUCERS that prepare the cost blocks of the
// next macro-step in LDS - on the matrix cores in fused mode, by copying from the stored cost
// tensor in unfused mode.  The roles are separate wavefronts, so that the producers' loads and
// their latency never sit in the consumer's instruction stream; the wavefronts of a band are
// placed on one SIMD (elected at run time from the hardware SIMD id; any placement is correct,
// this one keeps one consumer per SIMD).  One workgroup barrier per macro-step keeps them in step.
// Small problems use one band, or two consecutive bands of a pair, per workgroup (see below).
//
// Cells outside the N x M grid are not masked.  They are fed a huge finite cost (kBigCost) and the
// table boundary is a huge finite value (kBig) instead of +inf: a cell whose three neighbours are
// all kBig stays exactly kBig (kBig + kBigCost == kBig in float64), a grid cell sees
// (float)(kBig - m) = +inf and 2^-inf = 0 for such a neighbour, exactly as Sec. 2's boundary
// conditions R[i,0] = R[0,j] = +inf demand, and no inf - inf = NaN can arise.  Cells right of
// column M or below row N get finite garbage that no grid cell depends on.
//
// Cost values reach the lanes through an LDS ring indexed by STEP, not by column:
// cell (band row t, column j) lives at ring[t][(j + t) mod 128].  At step s every lane reads
// position s mod 128 of its own row, so the address of a step is a per-macro-step base plus an
// immediate.  Four phases of 32 steps exist: the one being read, the one still being flushed (E,
// backward) and the two being filled for later.  32x32 cost blocks are written with that skew.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_core.h"
#include "layout.h"

namespace sdtw {

constexpr int kPeekStep = 24;      // step of a macro-step at which the next boundary values are requested
constexpr int kRingCols = 128;     // four phases of 32 steps
constexpr int kRingStride = 129;   // floats per band row in LDS (odd: lanes hit distinct banks)
constexpr int kRingFloats = kBandRows * kRingStride;
// Workgroup shapes: SLOTS bands per workgroup, each with one consumer and NPROD producer wavefronts.
//   SLOTS=4, NPROD=1|2 (512|768 threads): large problems; the wavefronts of a band share a SIMD.
//   SLOTS=1, NPROD=1|2 (128|192 threads): small problems that cannot fill the chip anyway; the
//   wavefronts of a band land on different SIMDs, so producing the cost never delays the DP chain.
// Workgroup shapes: 1 band (consumer + producers), 4 bands of 4 pairs, or 2 consecutive bands of one
// pair ("chained": the upper band hands its last row to the lower one through LDS).  The chained
// shape with two producers per band has 8 wavefronts of which two stay unused, so that the two
// consumers (wavefronts 0 and 1) share their SIMD with nobody.
constexpr int wg_threads(int slots, int nprod) { return (slots == 2 && nprod == 2) ? 512 : slots * (1 + nprod) * 64; }
constexpr int kChainLag = 3;  // macro-steps the second band of a chained pair runs behind the first
// LDS hand-over ring of a chained pair: 4 phases of 32 edge values, then the slots the other lanes
// write to (see kEdgeOut below)
constexpr int kHandRing = 4 * kBlk;
constexpr int kHandDoubles = kHandRing + kBandRows + kBlk;
// Large problems (the 4-band workgroups) are bound by HBM traffic, of which the float64 table R would
// be the largest part (8 bytes per cell written, 8 read).  There the forward keeps only the lane
// state at the start of every macro-step (1/16 of R) and the backward recomputes each macro-step of
// R before it uses it - from the cost block that is in the ring anyway, in either mode.
constexpr bool dp_recompute(int /*kch*/, int slots) { return slots == 4; }
constexpr float kBigCost = 3.0e38f;  // cost of a cell outside the grid
constexpr int kStatusTimeoutDp = 6;  // SDTW_ERR_TIMEOUT

__device__ __forceinline__ double min_f64(double a, double b)
{
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

__device__ __forceinline__ double max_f64(double a, double b)
{
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// The DP tables are kept in units of gamma*ln2: every stored value is the paper's value times
// c2 = log2(e)/gamma, so that differences of table entries are base-2 exponents as they stand.
// In these units  softmin_gamma(a,b,c) = m - L  with  m = min(a,b,c) (float64) and
// L = log2(sum_k 2^{-(v_k - m)}) in [0, log2 3] (float32).
// (Sec. 2 Eq. 2, evaluated with the max-shift of Sec. 4.2; the term of the minimum is 2^0 = 1.)
// The two other terms: with lo = min(b,c), hi = max(b,c), either a is the minimum and they are
// lo-a and hi-a, or lo is and they are a-lo and hi-lo; both cases are |a-lo| and hi-m.
__device__ __forceinline__ void softmin3_parts(double a, double b, double c, double &m, float &L)
{
    const double lo = min_f64(b, c), hi = max_f64(b, c);
    m = min_f64(a, lo);
    const float t1 = (float)__builtin_fabs(a - lo);
    const float t2 = (float)(hi - m);
    const float S = 1.0f + __builtin_amdgcn_exp2f(-t1) + __builtin_amdgcn_exp2f(-t2);
    L = __builtin_amdgcn_logf(S);
}

__device__ __forceinline__ float comp4(const float4 &v, int c)
{
    return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

// ---------------------------------------------------------------------------------------------
// Boundary values between bands.  They travel through a buffer pre-filled with kSentinel; each
// value is published with one 64-bit device-scope atomic store, so it validates itself (no flag,
// no fence).  resolve_boundary polls until all needed lanes have a value (`bits` is what an
// earlier prefetch saw); a band gives up after p.spin_limit polls, records SDTW_ERR_TIMEOUT and
// never waits again; other bands notice the recorded status and stop waiting too, so every
// kernel exits.
// ---------------------------------------------------------------------------------------------
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

// ---------------------------------------------------------------------------------------------
// Producer side: cost blocks into the ring.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ floatx16 zero16()
{
    floatx16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    return z;
}

// Writes a 32x32 cost block given in MFMA accumulator layout (acc[i]: row 8*(i/4)+4*(lane>>5)+(i&3),
// column lane&31) into the step-indexed ring.  Block rows are band rows 32*rb .., columns 32*cb ..;
// entries outside the grid (or outside the window |i-j| <= w) become kBigCost, negative round-off is
// clamped to 0.
__device__ __forceinline__ void store_block_acc(float *ring, const floatx16 &acc, int rb, int cb, int row0, int N,
                                                int M, int w, int lane)
{
    const int h = lane >> 5, c = lane & 31;
    const int sbase = 32 * (cb + rb) + c + 4 * h;
    float *rowbase = ring + (32 * rb + 4 * h) * kRingStride;
    const int i0 = row0 + 32 * rb, j0 = 32 * cb;
    const bool inside = (i0 + 32 <= N) && (j0 >= 0) && (j0 + 32 <= M) && (j0 + 31 - i0 <= w) && (i0 + 31 - j0 <= w);
    // A lane's 16 entries sit at steps sbase + rr + (0..31); within the 128 ring positions they wrap
    // only in blocks that start in the last phase.  Everywhere else (and inside the grid and the
    // window) an entry's address is the lane's base plus a constant: nothing to compute per entry.
    const int phase = (cb + rb) & 3;
    if (inside && phase != 3) {
        float *lane_base = rowbase + (32 * phase + c + 4 * h);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rr = 8 * (i >> 2) + (i & 3);
            lane_base[rr * kRingStride + rr] = fmaxf(acc[i], 0.0f);
        }
        return;
    }
    const bool col_ok = (unsigned)(j0 + c) < (unsigned)M;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int rr = 8 * (i >> 2) + (i & 3);  // + 4h = row inside the block
        const int pos = (sbase + rr) & (kRingCols - 1);
        float v = fmaxf(acc[i], 0.0f);
        if (!inside) v = (col_ok && (i0 + 4 * h + rr < N) && in_window(i0 + 4 * h + rr, j0 + c, w)) ? v : kBigCost;
        rowbase[rr * kRingStride + pos] = v;
    }
}

// Unfused mode: the 32x32 block of the stored cost tensor (row length ld) as 4 float4 per lane
// (lane -> row (lane>>3) + 8*it of the block, columns 4*(lane&7) ..), kBigCost outside the N x M grid
// and outside the window |i-j| <= w (tiles of the cost tensor that lie outside it were never written).
__device__ __forceinline__ void load_cost_block(float4 (&v)[4], const float *__restrict__ cost_b, int rb, int cb,
                                                int row0, int N, int M, int ld, int w, bool vec_m, int lane)
{
    const int c4 = (lane & 7) * 4, j0 = 32 * cb;
    const int i0 = row0 + 32 * rb;
    const bool all_in = (j0 + 31 - i0 <= w) && (i0 + 31 - j0 <= w);
    const bool none_in = (j0 - (i0 + 31) > w) || (i0 - (j0 + 31) > w);
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = row0 + 32 * rb + (lane >> 3) + 8 * it;
        const int col = j0 + c4;
        float4 t = make_float4(kBigCost, kBigCost, kBigCost, kBigCost);
        if (row < N && col >= 0 && !none_in) {
            const float *q = cost_b + (size_t)row * ld + col;
            if (vec_m && col + 3 < M) {
                t = *reinterpret_cast<const float4 *>(q);
            } else {
                if (col + 0 < M) t.x = q[0];
                if (col + 1 < M) t.y = q[1];
                if (col + 2 < M) t.z = q[2];
                if (col + 3 < M) t.w = q[3];
            }
            if (!all_in) {
                t.x = in_window(row, col + 0, w) ? t.x : kBigCost;
                t.y = in_window(row, col + 1, w) ? t.y : kBigCost;
                t.z = in_window(row, col + 2, w) ? t.z : kBigCost;
                t.w = in_window(row, col + 3, w) ? t.w : kBigCost;
            }
        }
        v[it] = t;
    }
}

__device__ __forceinline__ void store_cost_block(float *ring, const float4 (&v)[4], int rb, int cb, int lane)
{
    const int c4 = (lane & 7) * 4;
    const int phase = (cb + rb) & 3;
    if (phase != 3) {  // no entry of the block wraps around the ring: constant offsets from the lane's base
        float *lane_base = ring + (32 * rb + (lane >> 3)) * kRingStride + 32 * phase + c4 + (lane >> 3);
#pragma unroll
        for (int it = 0; it < 4; ++it)
#pragma unroll
            for (int e = 0; e < 4; ++e) lane_base[8 * it * kRingStride + 8 * it + e] = comp4(v[it], e);
        return;
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = (lane >> 3) + 8 * it;
        float *rowp = ring + (32 * rb + r) * kRingStride;
        const int base = 32 * (cb + rb) + c4 + r;
#pragma unroll
        for (int e = 0; e < 4; ++e) rowp[(base + e) & (kRingCols - 1)] = comp4(v[it], e);
    }
}

// Any-D cost block straight from x and y (fused mode when D > 128).
__device__ __forceinline__ void generic_block(const Params &p, int b, float *ring, int rb, int cb, int row0, int lane)
{
    float out[16];
    const int i0 = row0 + 32 * rb, j0 = 32 * cb;
    cost_block(p, p.x + b * p.x_stride, p.y + b * p.y_stride, p.xn + b * p.xn_stride, p.yn + b * p.yn_stride,
               min(i0, p.N - 1), max(0, min(j0, p.M - 1)), lane, out);
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = out[i];
    // when the block origin had to be clamped the whole block lies outside the grid
    const bool origin_ok = (i0 < p.N) && (j0 >= 0) && (j0 < p.M);
    store_block_acc(ring, acc, rb, cb, row0, origin_ok ? p.N : 0, p.M, p.window, lane);
}

// The two cost blocks a macro-step `sg` must prepare for the following one.
//   forward  (DIR=+1): (lower rows, sg) then (upper rows, sg+1)
//   backward (DIR=-1): (upper rows, sg-2) then (lower rows, sg-3)
template <int DIR> __device__ __forceinline__ int blk_rb(int which) { return DIR > 0 ? 1 - which : which; }
template <int DIR> __device__ __forceinline__ int blk_cb(int sg, int which)
{
    return DIR > 0 ? sg + which : sg - 2 - which;
}

// Matrix-core producer for D <= 16*KG (KG = 1, 2, 4, 8 groups of 16 features).
//
// The inner products run on the fp16 matrix cores (v_mfma_f32_32x32x16_f16, float32 accumulate:
// 16 features per pass against 2 for the float32 matrix instruction, so three of them cost far
// less).  Float32 accuracy is kept by the split-half copies the prep kernel made: each scaled
// element is h1 + h2 (two float16), and <x_i,y_j> = (h1.k1 + h1.k2 + h2.k1) / (s_i s_j) up to
// ~2^-22 relative (Sec. 4.3 Eq. 8 supplies the norms; they are added in float32 afterwards).
// Lane (r = lane&31, h = lane>>5) holds features 16g+8h .. 16g+8h+7 of its row for group g; the
// copies are stored [row][group][piece][16] so that one row pointer plus immediates reaches all.
// The band's x pieces stay in registers for the whole sweep; y streams through NBUF stage
// buffers, each reloaded right after use with the data of the stage NBUF stages later.
// A producer makes the blocks W0 .. W0+NW-1 of the two blocks of each macro-step (NW = 2: both).

template <int KG, int DIR, int W0, int NW> struct HalfProducer {
    static constexpr int NST = NW * KG;                   // stages (one feature group of one block) per macro-step
    static constexpr int NBUF = NST < 8 ? NST : 8;        // stage buffers
    static_assert(NST % NBUF == 0, "stage buffers must divide the stages of a macro-step");
    static constexpr bool owns_rb(int rb) { return NW == 2 || rb == (DIR > 0 ? 1 - W0 : W0); }

    half8 xa[2][2][KG];     // [row block][piece][group]
    half8 ybuf[NBUF][2];    // [stage][piece]
    float yn_c[2], yis_c[2];  // ||y_c||^2 and 1/scale of this lane's column, for the blocks of the macro-step
    bool one_piece;         // the operands are float16 / bfloat16 values: their first piece is all of them (Params::pieces)

    __device__ __forceinline__ int ycol(const Params &p, int cb, int lane) const
    {
        const int col = 32 * cb + (lane & 31);
        return max(0, min(col, p.M - 1));
    }
    __device__ __forceinline__ void load_stage(const Params &p, const uint16_t *yh, int buf, int cb, int g, int lane)
    {
        const uint16_t *r = yh + (size_t)ycol(p, cb, lane) * (2 * p.Dp) + 8 * (lane >> 5) + 32 * g;
        ybuf[buf][0] = *reinterpret_cast<const half8 *>(r);
        if (!one_piece) ybuf[buf][1] = *reinterpret_cast<const half8 *>(r + 16);
    }
    // x pieces of the band, and the per-row table (||x_r||^2, -2/scale_r) in LDS
    __device__ __forceinline__ void init(const Params &p, const uint16_t *xh, const float *xnb, const float *xisb,
                                         float2 *rowtab, int row0, int lane)
    {
        one_piece = p.pieces == 1;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            if (!owns_rb(rb)) continue;
            const int row = min(row0 + 32 * rb + (lane & 31), p.N - 1);
            const uint16_t *r = xh + (size_t)row * (2 * p.Dp) + 8 * (lane >> 5);
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                xa[rb][0][g] = *reinterpret_cast<const half8 *>(r + 32 * g);
                xa[rb][1][g] = *reinterpret_cast<const half8 *>(r + 32 * g + 16);
            }
            if (lane < 32) rowtab[32 * rb + lane] = make_float2(xnb[row], -2.0f * xisb[row]);
        }
    }
    __device__ __forceinline__ floatx16 mfma3(floatx16 acc, int rb, int g, const half8 &k1, const half8 &k2) const
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[rb][0][g], k1, acc, 0, 0, 0);
        if (!one_piece) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[rb][0][g], k2, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[rb][1][g], k1, acc, 0, 0, 0);
        }
        return acc;
    }
    // acc (scaled inner products) -> cost block in the ring:  d = ||x||^2 + ||y||^2 - 2 <x,y>, clamped at 0
    __device__ __forceinline__ void finish(const Params &p, float *ring, const float2 *rowtab, floatx16 acc,
                                           int rb, int cb, float ync, float yisc, int row0, int lane) const
    {
        const int h = lane >> 5;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float2 t = rowtab[32 * rb + 8 * (i >> 2) + 4 * h + (i & 3)];
            acc[i] = fmaf(acc[i], t.y * yisc, t.x + ync);
        }
        store_block_acc(ring, acc, rb, cb, row0, p.N, p.M, p.window, lane);
    }
    // one whole block, loads included (start-up only)
    __device__ __forceinline__ void block_now(const Params &p, const uint16_t *yh, const float *ynb,
                                              const float *yisb, float *ring, const float2 *rowtab, int rb, int cb,
                                              int row0, int lane)
    {
        const int col = ycol(p, cb, lane);
        // goes through the stage buffers (NBUF >= KG) so that start-up needs no registers of its own
#pragma unroll
        for (int g = 0; g < KG; ++g) load_stage(p, yh, g, cb, g, lane);
        __builtin_amdgcn_sched_barrier(0);
        floatx16 acc = zero16();
#pragma unroll
        for (int g = 0; g < KG; ++g) acc = mfma3(acc, rb, g, ybuf[g][0], ybuf[g][1]);
        finish(p, ring, rowtab, acc, rb, cb, ynb[col], yisb[col], row0, lane);
        __builtin_amdgcn_sched_barrier(0);
    }
    // stage buffers and column norms for the first macro-step `sg`
    __device__ __forceinline__ void prime(const Params &p, const uint16_t *yh, const float *ynb, const float *yisb,
                                          int sg, int lane)
    {
#pragma unroll
        for (int q = 0; q < NBUF; ++q) load_stage(p, yh, q, blk_cb<DIR>(sg, W0 + q / KG), q % KG, lane);
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int col = ycol(p, blk_cb<DIR>(sg, W0 + i), lane);
            yn_c[i] = ynb[col];
            yis_c[i] = yisb[col];
        }
    }
    // the blocks of macro-step sg
    __device__ __forceinline__ void run(const Params &p, const uint16_t *yh, const float *ynb, const float *yisb,
                                        float *ring, const float2 *rowtab, int sg, int row0, int lane)
    {
        const int sgn = sg + DIR;  // next macro-step
        float nyn[2], nyis[2];
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int col = ycol(p, blk_cb<DIR>(sgn, W0 + i), lane);
            nyn[i] = ynb[col];
            nyis[i] = yisb[col];
        }
        auto reload = [&](int q) {  // refill the buffer of stage q with the stage NBUF stages later
            const int q2 = q + NBUF;
            if (q2 < NST)
                load_stage(p, yh, q % NBUF, blk_cb<DIR>(sg, W0 + q2 / KG), q2 % KG, lane);
            else
                load_stage(p, yh, q % NBUF, blk_cb<DIR>(sgn, W0 + (q2 - NST) / KG), (q2 - NST) % KG, lane);
        };
        // Reloads of the first half of a block's stages are issued right after their use; those of
        // the second half wait until the block has been written out, so that the epilogue's
        // temporaries and all in-flight stage buffers are never live together.
        constexpr int kEarly = KG > 1 ? KG / 2 : 1;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int which = W0 + w, rb = blk_rb<DIR>(which);
            floatx16 acc = zero16();
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                const int q = w * KG + g;
                acc = mfma3(acc, rb, g, ybuf[q % NBUF][0], ybuf[q % NBUF][1]);
                __builtin_amdgcn_sched_barrier(0);
                if (g < kEarly) reload(q);
            }
            finish(p, ring, rowtab, acc, rb, blk_cb<DIR>(sg, which), yn_c[w], yis_c[w], row0, lane);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = kEarly; g < KG; ++g) reload(w * KG + g);
        }
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            yn_c[i] = nyn[i];
            yis_c[i] = nyis[i];
        }
    }
};

// ---------------------------------------------------------------------------------------------
// Unfused cost tensor d[B,N,M] for D <= 16*KG on the fp16 matrix cores (Sec. 4.3 "unfused":
// computed once and stored), from the same split-half copies and with the same arithmetic as the
// fused producer.  One workgroup = 4 wavefronts = a 128-row x (32*CB)-column tile.  The y pieces of
// the tile's columns are brought into LDS once (coalesced 512-byte rows; the kernel is bound by
// operand traffic from L2, so no wavefront fetches what another one of its workgroup fetches); each
// wavefront keeps the pieces of its 32 rows in registers and walks the CB column blocks.
// LDS column stride 512+16 bytes: the 16-byte operand reads of 8 consecutive columns hit all banks.
// ---------------------------------------------------------------------------------------------
template <int KG> constexpr int cost_col_halfs() { return 32 * KG + 8; }
// floats per row of a wavefront's 32 x (32*CB) output tile while it waits in LDS to be stored row by row
template <int CB> constexpr int cost_stage_stride() { return 32 * CB + 4; }
template <int KG, int CB> constexpr int cost_lds_bytes()
{
    constexpr int operands = 32 * CB * cost_col_halfs<KG>() * 2, stage = 4 * 32 * cost_stage_stride<CB>() * 4;
    return operands > stage ? operands : stage;
}

// Second half of both cost-tensor kernels: the tile's inner products on the matrix cores, the cost
// from them (Sec. 4.3 Eq. 8), and the stores.  xa: the wavefront's 32 rows of x as operand pieces,
// xn_r / m2is_r: ||x||^2 and -2/scale of the 16 rows a lane's accumulator entries belong to, ys /
// ytab: the tile's columns of y in LDS (pieces; norm and 1/scale), lds: the same memory, reused for
// the stores once every wavefront has passed the barrier in here.
template <int KG, int CB>
__device__ __forceinline__ void cost_tile_finish(const Params &p, const half8 (&xa)[2][KG], const float (&xn_r)[16],
                                                 const float (&m2is_r)[16], const _Float16 *ys, const float2 *ytab,
                                                 unsigned char *lds, int b, int i0, int jbase, bool rows_live, int lane,
                                                 int w, int h)
{
    constexpr int kCol = cost_col_halfs<KG>();
    float *dst = p.cost + (size_t)b * p.N * p.M;
    floatx16 acc[CB];
#pragma unroll
    for (int cbk = 0; cbk < CB; ++cbk) {
        const _Float16 *yc = ys + (cbk * 32 + (lane & 31)) * kCol + 8 * h;
        acc[cbk] = zero16();
        if (rows_live && jbase + cbk * 32 < p.M) {
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                const half8 k1 = *reinterpret_cast<const half8 *>(yc + 32 * g);
                const half8 k2 = *reinterpret_cast<const half8 *>(yc + 32 * g + 16);
                acc[cbk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0][g], k1, acc[cbk], 0, 0, 0);
                if (p.pieces != 1) {  // (float16 / bfloat16 inputs: the first piece is the whole element)
                    acc[cbk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[0][g], k2, acc[cbk], 0, 0, 0);
                    acc[cbk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[1][g], k1, acc[cbk], 0, 0, 0);
                }
            }
            const float2 yt = ytab[cbk * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[cbk][i] = fmaxf(fmaf(acc[cbk][i], m2is_r[i] * yt.y, xn_r[i] + yt.x), 0.0f);
        }
    }
    if (!p.vec_m) {  // rows of the tensor are not 16-byte aligned: element stores straight from the accumulators
        if (rows_live) {
#pragma unroll
            for (int cbk = 0; cbk < CB; ++cbk) {
                const int col = jbase + cbk * 32 + (lane & 31);
                if (col < p.M) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = i0 + acc_row(i, lane);
                        if (row < p.N) __builtin_nontemporal_store(acc[cbk][i], &dst[(size_t)row * p.M + col]);
                    }
                }
            }
        }
        return;
    }
    // An accumulator holds one column of 16 rows per lane; stored like that, an instruction touches 32
    // rows with 4 bytes each.  The wavefront's 32 x (32*CB) tile goes through LDS instead (the operand
    // area, once every wavefront has finished reading it) and leaves as whole rows, 16 bytes per lane.
    __syncthreads();
    constexpr int kStage = cost_stage_stride<CB>();
    float *stage = reinterpret_cast<float *>(lds) + w * (32 * kStage);
#pragma unroll
    for (int cbk = 0; cbk < CB; ++cbk)
#pragma unroll
        for (int i = 0; i < 16; ++i) stage[acc_row(i, lane) * kStage + cbk * 32 + (lane & 31)] = acc[cbk][i];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (!rows_live) return;
    constexpr int kVecPerRow = 8 * CB;  // float4 per tile row
#pragma unroll
    for (int k = 0; k < (32 * kVecPerRow) / 64; ++k) {
        const int idx = k * 64 + lane;
        const int r = idx / kVecPerRow, c4 = (idx % kVecPerRow) * 4;
        typedef float floatx4 __attribute__((ext_vector_type(4)));
        const floatx4 v = *reinterpret_cast<const floatx4 *>(stage + r * kStage + c4);
        const int row = i0 + r, col = jbase + c4;
        if (row < p.N && col < p.M)
            __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(&dst[(size_t)row * p.M + col]));
    }
}

template <int KG, int CB>
__global__ __launch_bounds__(256) void cost_tensor_half_kernel(Params p)
{
    constexpr int kCol = cost_col_halfs<KG>();
    __shared__ __attribute__((aligned(16))) unsigned char lds[cost_lds_bytes<KG, CB>()];
    __shared__ float2 ytab[32 * CB];  // (||y_j||^2, 1/scale_j)
    _Float16 *ys = reinterpret_cast<_Float16 *>(lds);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, h = lane >> 5;
    const int b = blockIdx.z;
    const int i0 = blockIdx.y * 128 + w * 32;
    const uint16_t *xh = p.xh + b * p.xh_stride, *yh = p.yh + b * p.yh_stride;
    const float *xnb = p.xn + b * p.xn_stride, *ynb = p.yn + b * p.yn_stride;
    const float *xisb = p.xis + b * p.xn_stride, *yisb = p.yis + b * p.yn_stride;
    const int jbase = blockIdx.x * (32 * CB);
    {   // no cell of the 128 x 32*CB tile inside the window: nothing to compute (the sweeps never read it)
        const int ti0 = blockIdx.y * 128;
        if (jbase - (ti0 + 127) > p.window || ti0 - (jbase + 32 * CB - 1) > p.window) return;
    }

    // y pieces of the tile's columns -> LDS: a column is 4*KG chunks of 16 bytes
    constexpr int kChunks = 4 * KG;
    for (int e = tid; e < 32 * CB * kChunks; e += 256) {
        const int c = e / kChunks, ch = e % kChunks;
        const int colc = min(jbase + c, p.M - 1);
        const half8 v = *reinterpret_cast<const half8 *>(yh + (size_t)colc * (2 * p.Dp) + 8 * ch);
        *reinterpret_cast<half8 *>(&ys[c * kCol + 8 * ch]) = v;
    }
    if (tid < 32 * CB) {
        const int colc = min(jbase + tid, p.M - 1);
        ytab[tid] = make_float2(ynb[colc], yisb[colc]);
    }
    // own rows' pieces -> registers
    half8 xa[2][KG];
    float xn_r[16], m2is_r[16];
    const bool rows_live = i0 < p.N;
    {
        const int row = min(i0 + (lane & 31), p.N - 1);
        const uint16_t *r = xh + (size_t)row * (2 * p.Dp) + 8 * h;
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            xa[0][g] = *reinterpret_cast<const half8 *>(r + 32 * g);
            xa[1][g] = *reinterpret_cast<const half8 *>(r + 32 * g + 16);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rr = min(i0 + acc_row(i, lane), p.N - 1);
            xn_r[i] = xnb[rr];
            m2is_r[i] = -2.0f * xisb[rr];
        }
    }
    __syncthreads();

    cost_tile_finish<KG, CB>(p, xa, xn_r, m2is_r, ys, ytab, lds, b, i0, jbase, rows_live, lane, w, h);
}

// The same with the start of the forward call folded in (unfused mode without band constraint or
// length vectors, rows of 16-byte aligned float4): one launch instead of forward_prep_kernel and
// cost_tensor_half_kernel, which for small problems are two chains of memory round trips of about
// equal length.  Every workgroup makes the norms, scales and split-half pieces of its own 128 rows
// of x (in registers, already in the layout of the matrix operand) and of its 32*CB rows of y (into
// LDS) from x and y themselves - the rows of a tile are split again by every tile that shares them,
// which costs less than the launch it saves - and the workgroups of the first tile column / row also
// leave them in the workspace for the later kernels.  Header, tickets and the "not written yet"
// marks of the boundary rows are spread over all workgroups.
template <int KG, int CB>
__global__ __launch_bounds__(256) void cost_tensor_prep_kernel(Params p)
{
    constexpr int kCol = cost_col_halfs<KG>();
    constexpr int kDp = 16 * KG;
    __shared__ __attribute__((aligned(16))) unsigned char lds[cost_lds_bytes<KG, CB>()];
    __shared__ float2 ytab[32 * CB];  // (||y_j||^2, 1/scale_j)
    __shared__ float2 xtab[128];      // (||x_i||^2, -2/scale_i) of the tile's rows
    _Float16 *ys = reinterpret_cast<_Float16 *>(lds);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, h = lane >> 5;
    const int b = blockIdx.z;
    const int i0 = blockIdx.y * 128 + w * 32;
    const int jbase = blockIdx.x * (32 * CB);
    const float *xb = p.x + b * p.x_stride, *yb = p.y + b * p.y_stride;

    // start of the call
    const size_t nblk = (size_t)gridDim.x * gridDim.y * gridDim.z;
    const size_t blk = ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (tid == 0 && blk == 0) stamp_header(p);
    fill_boundary_rows(p, p.brow, false, blk, nblk);
    if (p.two_sweep) fill_boundary_rows(p, p.brow_b, true, blk, nblk);

    // (the loads of the x rows are asked for together with those of the y rows: one round trip for both)
    const int xr_row = min(i0 + (lane & 31), p.N - 1);
    float xv[KG][8];
    {
        const float *xr = xb + (size_t)xr_row * p.D;
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            const int k = 16 * g + 8 * h;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
            if (k < p.D) a = *reinterpret_cast<const float4 *>(xr + k);
            if (k + 4 < p.D) c = *reinterpret_cast<const float4 *>(xr + k + 4);
            xv[g][0] = a.x; xv[g][1] = a.y; xv[g][2] = a.z; xv[g][3] = a.w;
            xv[g][4] = c.x; xv[g][5] = c.y; xv[g][6] = c.z; xv[g][7] = c.w;
        }
    }
    // y rows of the tile's columns, one block of 32 per wavefront (wavefront w takes blocks w, w+4, ...):
    // like the x rows, half a row per lane, so that a row's maximum and norm take one exchange
    for (int cbk = w; cbk < CB; cbk += 4) {
        const int c = cbk * 32 + (lane & 31);
        const int col = min(jbase + c, p.M - 1);
        const float *yr = yb + (size_t)col * p.D;
        float yv[KG][8];
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            const int k = 16 * g + 8 * h;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c2 = a;
            if (k < p.D) a = *reinterpret_cast<const float4 *>(yr + k);
            if (k + 4 < p.D) c2 = *reinterpret_cast<const float4 *>(yr + k + 4);
            yv[g][0] = a.x; yv[g][1] = a.y; yv[g][2] = a.z; yv[g][3] = a.w;
            yv[g][4] = c2.x; yv[g][5] = c2.y; yv[g][6] = c2.z; yv[g][7] = c2.w;
        }
        float acc = 0.f, mx = 0.f;
#pragma unroll
        for (int g = 0; g < KG; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                acc = fmaf(yv[g][e], yv[g][e], acc);
                mx = fmaxf(mx, fabsf(yv[g][e]));
            }
        acc += __shfl_xor(acc, 32);  // the other half of the row
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sc, inv;
        split_scale(mx, sc, inv);
        if (h == 0) ytab[c] = make_float2(acc, inv);
        const bool owner = blockIdx.y == 0 && jbase + c < p.M;  // leaves them in the workspace
        if (owner && h == 0) {
            p.yn[b * p.yn_stride + col] = acc;
            p.yis[b * p.yn_stride + col] = inv;
        }
        uint16_t *dsth = p.yh + b * p.yh_stride + (size_t)col * (2 * kDp) + 8 * h;
#pragma unroll
        for (int g = 0; g < KG; ++g) {
            half8 h1, h2;
            split8(yv[g], sc, h1, h2);
            *reinterpret_cast<half8 *>(&ys[c * kCol + 32 * g + 8 * h]) = h1;  // [group of 16 features][piece][16]
            *reinterpret_cast<half8 *>(&ys[c * kCol + 32 * g + 8 * h + 16]) = h2;
            if (owner) {
                *reinterpret_cast<half8 *>(dsth + 32 * g) = h1;
                *reinterpret_cast<half8 *>(dsth + 32 * g + 16) = h2;
            }
        }
    }
    // own rows of x, straight into the operand layout: lane (r, h) holds features 16g+8h .. +7 of row r
    half8 xa[2][KG];
    const bool rows_live = i0 < p.N;
    {
        const int r = lane & 31;
        const int row = xr_row;
        float acc = 0.f, mx = 0.f;
#pragma unroll
        for (int g = 0; g < KG; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                acc = fmaf(xv[g][e], xv[g][e], acc);
                mx = fmaxf(mx, fabsf(xv[g][e]));
            }
        acc += __shfl_xor(acc, 32);  // the other half of the row
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sc, inv;
        split_scale(mx, sc, inv);
#pragma unroll
        for (int g = 0; g < KG; ++g) split8(xv[g], sc, xa[0][g], xa[1][g]);
        if (h == 0) xtab[w * 32 + r] = make_float2(acc, -2.0f * inv);
        if (blockIdx.x == 0 && i0 + r < p.N) {  // this tile column leaves them in the workspace
            if (h == 0) {
                p.xn[b * p.xn_stride + row] = acc;
                p.xis[b * p.xn_stride + row] = inv;
            }
            uint16_t *dsth = p.xh + b * p.xh_stride + (size_t)row * (2 * kDp) + 8 * h;
#pragma unroll
            for (int g = 0; g < KG; ++g) {
                *reinterpret_cast<half8 *>(dsth + 32 * g) = xa[0][g];
                *reinterpret_cast<half8 *>(dsth + 32 * g + 16) = xa[1][g];
            }
        }
    }
    __syncthreads();
    float xn_r[16], m2is_r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float2 t = xtab[w * 32 + acc_row(i, lane)];
        xn_r[i] = t.x;
        m2is_r[i] = t.y;
    }

    cost_tile_finish<KG, CB>(p, xa, xn_r, m2is_r, ys, ytab, lds, b, i0, jbase, rows_live, lane, w, h);
}

// ---------------------------------------------------------------------------------------------
// Workgroup bookkeeping shared by both kernels.
// ---------------------------------------------------------------------------------------------
template <int SLOTS> struct WgShared {
    float ring[SLOTS][kRingFloats];
    double edge_in[SLOTS][kBlk];  // boundary values of the current macro-step, one per step
    double ftop[SLOTS][kBlk];     // backward with recomputation: the forward's row above the band
    float2 rowtab[SLOTS][kBandRows];  // per band row: (||x_r||^2, -2/scale_r) for the cost epilogue
    int simd_count[4];
    int blk_dead[SLOTS][2];  // reverse sweep: the E blocks completed by macro-step sg hold no non-zero (indexed by sg & 1)
};

// Values the band's edge row (last row in the forward sweep, first in the reverse sweep) produced
// in the current macro-step, one per step, for the neighbouring band: double[SLOTS][kEdgeOut] in
// LDS.  Every lane writes its value each step; only the edge lane's address points into [0,32),
// the others write to slots of their own behind it.  (Kept as an object of its own, so that these
// stores are known not to touch the ring or the incoming boundary values.)
constexpr int kEdgeOut = kBlk + kBandRows + kBlk;

// Groups the wavefronts that share a SIMD as consumer (0) and producers (1, 2) of one band slot.
// If the wavefronts are not spread evenly over the SIMDs, falls back to wavefront w -> role w/4,
// slot w%4.
__device__ __forceinline__ void elect_role(WgShared<4> &sh, int lane, int w, int per_simd, int &producer, int &slot)
{
    if (threadIdx.x < 4) sh.simd_count[threadIdx.x] = 0;
    __syncthreads();
    const unsigned hwid = __builtin_amdgcn_s_getreg((1 << 11) | (4 << 6) | 4);  // HW_ID bits [5:4]: SIMD id
    const int simd = (int)(hwid & 3u);
    int idx = 0;
    if (lane == 0) idx = atomicAdd(&sh.simd_count[simd], 1);
    idx = __builtin_amdgcn_readfirstlane(idx);
    __syncthreads();
    const bool even = sh.simd_count[0] == per_simd && sh.simd_count[1] == per_simd && sh.simd_count[2] == per_simd &&
                      sh.simd_count[3] == per_simd;
    producer = __builtin_amdgcn_readfirstlane(even ? idx : (w >> 2));
    slot = __builtin_amdgcn_readfirstlane(even ? simd : (w & 3));
}

// Roles in a chained pair: wavefronts 0, 1 are the consumers of the pair's first and second band,
// 2, 3 their (first) producers, 6, 7 their second producers; 4, 5 stay unused.  Wavefront i of a
// workgroup lands on SIMD i mod 4, so each consumer has a SIMD to itself.
__device__ __forceinline__ void chain_role(int w, int &producer, int &slot)
{
    slot = w & 1;
    const int r = w >> 1;
    producer = r == 0 ? 0 : (r == 1 ? 1 : (r == 3 ? 2 : -1));
}

// ---------------------------------------------------------------------------------------------
// Forward DP (Sec. 2 Eq. 1-2 in the anti-diagonal order of Sec. 4.1).
// Workgroups take tickets in band-major order: a band only ever waits for a band with a smaller
// ticket, which is running or done, so the wait ends whatever order the hardware starts
// workgroups in.  The table goes to HBM step-major, R[b][band][s][lane]: one coalesced 512-byte
// store per step; the band's last row goes to the boundary buffer.
//   KCH > 0: fused, D <= 16*KCH (fp16 matrix cores, split-half operands);  KCH == 0: fused, any D
//   (float32 from x and y);  KCH < 0: unfused.
// ---------------------------------------------------------------------------------------------
template <int KCH, int SLOTS, int NPROD>
__device__ __forceinline__ void forward_dp_body(const Params &p, float *__restrict__ value, WgShared<SLOTS> &sh,
                                                unsigned &ticket_s, double (&edge_out)[SLOTS][kEdgeOut],
                                                double (&hand)[kHandDoubles])
{
    static_assert(SLOTS == 4 || SLOTS == 2 || SLOTS == 1, "supported workgroup shapes");
    static_assert(NPROD == 1 || (NPROD == 2 && KCH > 0), "two producers only split MFMA work");
    constexpr int kThreads = wg_threads(SLOTS, NPROD);
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (threadIdx.x == 0) ticket_s = atomicAdd(&p.hdr->fwd_ticket, 1u);
    for (int e = threadIdx.x; e < SLOTS * kRingFloats; e += kThreads) (&sh.ring[0][0])[e] = kBigCost;
    int producer, slot;  // producer: 0 = consumer, 1.. = producer number
    if constexpr (SLOTS == 4) {
        elect_role(sh, lane, w, 1 + NPROD, producer, slot);  // contains two barriers
    } else if constexpr (SLOTS == 2) {
        for (int e = threadIdx.x; e < kHandDoubles; e += kThreads) hand[e] = kBig;
        chain_role(w, producer, slot);
        __syncthreads();
    } else {
        producer = w;
        slot = 0;
        __syncthreads();
    }
    const unsigned ticket = __builtin_amdgcn_readfirstlane(ticket_s);
    int k, b;
    // The macro-steps to run, [rg.lo, rg.hi], follow from the ticket alone, so that every wavefront
    // of the workgroup passes the same number of barriers.
    SweepRange rg;
    if constexpr (SLOTS == 2) {  // ticket -> (pair of bands, pair of sequences); the slot is the band of the pair
        const int kp = ticket / (unsigned)p.B;
        b = ticket - kp * p.B;
        k = 2 * kp + (slot & 1);
        rg = sweep_range(p, 2 * kp * kBandRows, min(2 * kp + 1, p.nbands - 1) * kBandRows, pair_len(p.x_len, b, p.N),
                         pair_len(p.y_len, b, p.M));
    } else {
        const int ngroups = (p.B + SLOTS - 1) / SLOTS;
        k = ticket / (unsigned)ngroups;
        const int b0 = (ticket - k * ngroups) * SLOTS;
        b = b0 + slot;
        int nl = 1, ml = 1;  // the longest sequences among the workgroup's pairs
        for (int s2 = 0; s2 < SLOTS; ++s2) {
            if (b0 + s2 < p.B) {
                nl = max(nl, pair_len(p.x_len, b0 + s2, p.N));
                ml = max(ml, pair_len(p.y_len, b0 + s2, p.M));
            }
        }
        rg = sweep_range(p, k * kBandRows, k * kBandRows, nl, ml);
    }
    const bool live = (k < p.nbands) && (b < p.B) && rg.hi >= rg.lo;
    // chained pair: the second band does macro-step sg in workgroup iteration sg - rg.lo + kChainLag
    const int lag = (SLOTS == 2) ? kChainLag * slot : 0;
    const int niter = max(rg.hi - rg.lo + 1, 0) + ((SLOTS == 2) ? kChainLag : 0);
    if constexpr (SLOTS == 2) {
        if (producer < 0) {  // unused wavefront: only keeps the barrier count (one before the loop, one per iteration)
            for (int it = 0; it <= niter; ++it) __syncthreads();
            return;
        }
    }

    const int M = p.M, N = p.N;
    const int row0 = k * kBandRows;
    float *ring = sh.ring[slot];
    const int bb = live ? b : 0;
    // The pair's own lengths (ragged batches): cells beyond them are outside the grid for the cost
    // producers (cost kBigCost), which is all it takes - their table entries are huge, their E is 0.
    const int Nl = pair_len(p.x_len, bb, N), Ml = pair_len(p.y_len, bb, M);
    Params pl = p;
    pl.N = Nl;
    pl.M = Ml;
    [[maybe_unused]] const float *xb = p.x + bb * p.x_stride, *yb = p.y + bb * p.y_stride;
    const float *xnb = p.xn + bb * p.xn_stride, *ynb = p.yn + bb * p.yn_stride;
    const float *xisb = p.xis + bb * p.xn_stride, *yisb = p.yis + bb * p.yn_stride;
    const uint16_t *xh = p.xh + bb * p.xh_stride, *yh = p.yh + bb * p.yh_stride;
    float2 *rowtab = sh.rowtab[slot];

    if (producer) {
        // ------------------------------------------------------------------ producer wavefront
        if constexpr (KCH > 0 && NPROD == 2) {
            // producer 1 makes (lower rows, sg), producer 2 makes (upper rows, sg+1)
            auto body = [&](auto &mp, bool first_block) {
                if (live) {
                    mp.init(pl, xh, xnb, xisb, rowtab, row0, lane);
                    if (first_block) mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 0, rg.lo, row0, lane);
                    mp.prime(pl, yh, ynb, yisb, rg.lo, lane);
                }
                __syncthreads();
                for (int it = 0; it < niter; ++it) {
                    const int sg = rg.lo + it - lag;
                    if (live && sg >= rg.lo && sg <= rg.hi) mp.run(pl, yh, ynb, yisb, ring, rowtab, sg, row0, lane);
                    __syncthreads();
                }
            };
            if (producer == 1) {
                HalfProducer<KCH, +1, 0, 1> mp;
                body(mp, false);
            } else {
                HalfProducer<KCH, +1, 1, 1> mp;
                body(mp, true);
            }
        } else if constexpr (KCH > 0) {
            HalfProducer<KCH, +1, 0, 2> mp;
            if (live) {
                mp.init(pl, xh, xnb, xisb, rowtab, row0, lane);
                mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 0, rg.lo, row0, lane);  // (upper rows, first column block)
                mp.prime(pl, yh, ynb, yisb, rg.lo, lane);
            }
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = rg.lo + it - lag;
                if (live && sg >= rg.lo && sg <= rg.hi) mp.run(pl, yh, ynb, yisb, ring, rowtab, sg, row0, lane);
                __syncthreads();
            }
        } else if constexpr (KCH == 0) {
            if (live) generic_block(pl, b, ring, 0, rg.lo, row0, lane);
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = rg.lo + it - lag;
                if (live && sg >= rg.lo && sg <= rg.hi) {
                    generic_block(pl, b, ring, 1, sg, row0, lane);
                    generic_block(pl, b, ring, 0, sg + 1, row0, lane);
                }
                __syncthreads();
            }
        } else {
            const float *cost_b = p.cost + (size_t)bb * N * M;
            float4 pre[2][4];
            if (live) {
                load_cost_block(pre[0], cost_b, 0, rg.lo, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                store_cost_block(ring, pre[0], 0, rg.lo, lane);
                load_cost_block(pre[0], cost_b, 1, rg.lo, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                load_cost_block(pre[1], cost_b, 0, rg.lo + 1, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
            }
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = rg.lo + it - lag;
                if (live && sg >= rg.lo && sg <= rg.hi) {
                    store_cost_block(ring, pre[0], 1, sg, lane);
                    store_cost_block(ring, pre[1], 0, sg + 1, lane);
                    load_cost_block(pre[0], cost_b, 1, sg + 1, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                    load_cost_block(pre[1], cost_b, 0, sg + 2, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                }
                __syncthreads();
            }
        }
        return;
    }

    // ---------------------------------------------------------------------- consumer wavefront
    // The chain of dependent steps is what everything waits for: where this wavefront shares its SIMD
    // with producers, its instructions go first.
    __builtin_amdgcn_s_setprio(3);
    // CH: -1 = both neighbouring bands are reached through memory; 0 = the band below is the other
    // band of this workgroup (edge values go to the LDS hand-over ring); 1 = the band above is.
    // (Separate instances, so that each one reads and writes distinct LDS objects.)
    auto consume = [&](auto chain_c) {
    constexpr int CH = decltype(chain_c)::value;
    const double c2d = p.c2d;  // log2(e)/gamma
    bool gave_up = false;
    double left = kBig;                                  // R[i][j-1]
    double diag = (k == 0 && lane == 0) ? 0.0 : kBig;    // R[i-1][j-1]; R[0,0] = 0 in the paper's indexing
    const int kc = live ? k : 0;
    const unsigned long long *brow_in = p.brow + ((size_t)bb * p.nbands + (kc > 0 ? kc - 1 : 0)) * M;
    unsigned long long *brow_out = p.brow + ((size_t)bb * p.nbands + kc) * M;
    // RECOMP: the table is not stored; only the lane state at the start of every macro-step is
    // (checkpoints), and the backward kernel recomputes each macro-step of R from it.
    constexpr bool RECOMP = dp_recompute(KCH, SLOTS);
    // (table pointers are those of the band's macro-step 0; the table starts at macro-step table_base)
    const ptrdiff_t tb = table_base(p, kc);
    double *Rk = RECOMP ? nullptr : p.R + (((size_t)bb * p.nbands + kc) * (size_t)p.nm_tab - tb) * kBlk * kBandRows;
    double *Ck = RECOMP ? p.ckpt + (((size_t)bb * p.nbands + kc) * (size_t)p.nm_tab - tb) * 2 * kBandRows : nullptr;
    const int s_fin = (live && row0 + lane == Nl - 1) ? (Ml - 1 + lane) : -1;  // step of the pair's last cell
    const bool last_band = live && (k == (Nl - 1) / kBandRows);
    double fin = 0.0;
    const bool has_above = live && k > 0 && CH != 1;                // through memory
    const bool emit_bottom = live && (k + 1 < p.nbands);             // the band's last row goes to memory
    const float *my_ring = ring + lane * kRingStride;
    double *top = sh.edge_in[slot];
    double *eo = edge_out[slot];

    // row above the band for the first macro-step: lane l < 32 brings column 32*rg.lo + l
    // (the cells left of it are outside the grid or outside the window: the lane state starts as kBig)
    if constexpr (CH != 1) {
        double t0 = kBig;
        if (has_above) {
            const int j0 = rg.lo * kBlk + lane;
            const bool need = lane < kBlk && j0 < M;
            t0 = resolve_boundary(p, brow_in, j0, need, lane, gave_up, peek_boundary(brow_in, j0, need));
        }
        if (lane < kBlk) top[lane] = t0;
    }
    __syncthreads();

    for (int it = 0; it < niter; ++it) {
        const int sg = rg.lo + it - lag;
        if (live && sg >= rg.lo && sg <= rg.hi) {
            unsigned long long nxt_bits = (unsigned long long)__double_as_longlong(kBig);
            const int jn = (sg + 1) * kBlk + lane;
            const bool need_n = has_above && lane < kBlk && jn < M;
            const float *rd = my_ring + (sg & 3) * kBlk;
            // the macro-step's 32 cost values, read in one batch: read one per step they sit between the
            // steps' LDS stores, which they may not overtake, and each costs the chain a wait
            float dcv[kBlk];
#pragma unroll
            for (int u = 0; u < kBlk; ++u) dcv[u] = rd[u];
            // The row above, column 32*sg + u at step u: from the incoming boundary values, or from
            // the hand-over ring, where the band above put column c at slot (c + 63) mod 128.
            const double *top0 = top, *top1 = top + 1;  // step 0, steps 1..31
            if constexpr (CH == 1) {
                top0 = hand + ((sg + 1) & 3) * kBlk + (kBlk - 1);
                top1 = hand + ((sg + 2) & 3) * kBlk;
            }
            // Where this macro-step's values go: lane 63's are the band's last row (column
            // 32*sg + u - 63 at step u), the other lanes write to slots of their own.
            double *my_eo = eo + ((lane == kBandRows - 1) ? 0 : kBlk + lane);
            if constexpr (CH == 0) my_eo = hand + ((lane == kBandRows - 1) ? (sg & 3) * kBlk : kHandRing + lane);
            double *Rs = RECOMP ? nullptr : Rk + (size_t)sg * kBlk * kBandRows;
            if constexpr (RECOMP) {
                __builtin_nontemporal_store(left, &Ck[((size_t)sg * 2 + 0) * kBandRows + lane]);
                __builtin_nontemporal_store(diag, &Ck[((size_t)sg * 2 + 1) * kBandRows + lane]);
            }
            auto steps = [&](auto capture) {
#pragma unroll
                for (int u = 0; u < kBlk; ++u) {
                    // ask for the next macro-step's row above about one memory round trip before it
                    // is needed: asked earlier, the answer would be "not written yet" too often
                    if (u == kPeekStep && has_above) nxt_bits = peek_boundary(brow_in, jn, need_n);
                    const double up = lane_shr1(left, u == 0 ? top0[0] : top1[u - 1]);  // R[i-1][j]; lane 0 takes the row above the band
                    const float dc = dcv[u];
                    double m;
                    float L;
                    softmin3_parts(diag, up, left, m, L);
                    // every addition that builds the table is float64: a float32 rounding here would
                    // differ between the two sweeps and add up along the alignment path
                    const double cur = fma((double)dc, c2d, m) - (double)L;
                    if constexpr (!RECOMP)  // streamed once: keep it out of the caches
                        __builtin_nontemporal_store(cur, &Rs[u * kBandRows + lane]);
                    if constexpr (decltype(capture)::value) fin = (sg * kBlk + u == s_fin) ? cur : fin;
                    my_eo[u] = cur;  // lane 63: value of column 32*sg + u - 63 for the band below
                    diag = up;
                    left = cur;
                }
            };
            if (RECOMP && last_band)
                steps(std::true_type{});
            else
                steps(std::false_type{});
            // last row of the band: lanes 32..63 publish columns 32*sg - 63 + (lane - 32)
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            if (emit_bottom && lane >= kBlk) {
                const int j = sg * kBlk + lane - kBlk - (kBandRows - 1);
                // (a chained pair's upper band hands the row over through LDS; it still leaves it in
                // memory, where alignment_kernel looks for the columns that can hold a non-zero E)
                const double *src = (CH == 0) ? hand + (sg & 3) * kBlk : eo;
                if (j >= 0 && j < M) publish_boundary(brow_out, j, src[lane - kBlk]);
            }
            if constexpr (CH != 1) {
                double tn = kBig;
                if (has_above) tn = resolve_boundary(p, brow_in, jn, need_n, lane, gave_up, nxt_bits);
                if (lane < kBlk) top[lane] = tn;
            }
        }
        __syncthreads();
    }

    // R[N,M] of the pair: cell (N-1, M-1) was stored at step M-1+lane by the lane that owns row N-1
    if (live && row0 + lane == Nl - 1) {
        const double r = RECOMP ? fin : Rk[(size_t)(Ml - 1 + lane) * kBandRows + lane];
        p.rfinal[b] = r;                     // table units, for the backward sweep
        value[b] = (float)(r * p.inv_c2d);   // the paper's units
    }
    };
    if constexpr (SLOTS == 2) {
        if (slot == 0)
            consume(std::integral_constant<int, 0>{});
        else
            consume(std::integral_constant<int, 1>{});
    } else {
        consume(std::integral_constant<int, -1>{});
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
// E replaces the consumed cost value in the ring; the producers write it out as row-major 32x32
// blocks, with one flag byte per block saying whether any entry is non-zero.
// ---------------------------------------------------------------------------------------------
// A sweep may run macro-steps rg.lo .. rg.hi only (band constraint, per-pair lengths, or the columns
// alignment_kernel found to matter).  Block (rb, cb) of the band holds cells of macro-steps cb+rb and
// cb+rb+1: it is written out if both lie in [rg.lo, rg.hi_u] and it has a column inside the pair's
// grid; otherwise E is zero in all of it and the block is left alone with its flag cleared (nobody
// reads a block whose flag is clear).
__device__ __forceinline__ bool block_in_range(const SweepRange &rg, int rb, int cb)
{
    return cb + rb >= rg.lo && cb + rb + 1 <= rg.hi_u && cb <= rg.cb_last;
}

// idxb != nullptr: compact E.  A block that holds a non-zero takes the next free block of the pool
// (p.pool, handed out by an atomic counter in the workspace header) and leaves its number in the
// pair's block index idxb, which backward_prep_kernel pre-set to -1 = "all zero" everywhere; a block
// that finds the pool full raises the overflow flag instead (the backward call then redoes the
// gradients with the contracting sweep).
template <int COLS = kRingCols, int STRIDE = kRingStride>
__device__ __forceinline__ void flush_E_block(const Params &p, const SweepRange &rg, const float *ring,
                                              float *__restrict__ Eb, unsigned char *__restrict__ nzb, int rb, int cb,
                                              int row0, int lane, bool known_zero = false, int ring_row0 = 0,
                                              int32_t *__restrict__ idxb = nullptr)
{
    // ring_row0: the band row that the ring's first row holds (0, or 32 for a ring of the lower block row alone)
    if (cb < 0 || cb >= p.ncb || row0 + 32 * rb >= p.N || !block_in_range(rg, rb, cb)) return;
    if (known_zero) {  // the consumer found that no cell of the block's two macro-steps can be non-zero
        if (lane == 0) nzb[(size_t)(row0 / kBlk + rb) * p.ncb + cb] = 0;
        return;
    }
    const int c4 = (lane & 7) * 4, j0 = cb * kBlk;
    // the block's steps wrap around the ring only when it starts in the ring's last phase
    const int phase = (cb + rb) & (COLS / kBlk - 1);
    const bool nowrap = phase != COLS / kBlk - 1;
    auto read4 = [&](int it, float (&v)[4]) {
        const int r = (lane >> 3) + 8 * it;
        const float *rowp = ring + (32 * rb + r - ring_row0) * STRIDE;
        if (nowrap) {  // constant offsets from the lane's position
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = rowp[32 * phase + c4 + r + e];
        } else {
            const int base = 32 * (cb + rb) + c4 + r;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = rowp[(base + e) & (COLS - 1)];
        }
    };
    // First: does the block hold a non-zero inside the grid?  If not, only its flag is written: a
    // block with a clear flag is all zero by definition and is never read (for small gamma that is
    // almost every block).
    bool any = false;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        float v[4];
        read4(it, v);
        const int row = row0 + rb * 32 + (lane >> 3) + 8 * it;
        if (row < p.N) {
#pragma unroll
            for (int e = 0; e < 4; ++e) any |= (j0 + c4 + e < p.M) && v[e] != 0.f;
        }
    }
    const bool blk_any = __any(any);
    const size_t blk_id = (size_t)(row0 / kBlk + rb) * p.ncb + cb;
    if (idxb != nullptr) {
        unsigned slot = 0;
        if (blk_any && lane == 0) slot = atomicAdd(&p.hdr->pool_count, 1u);
        slot = (unsigned)__builtin_amdgcn_readfirstlane((int)slot);
        const bool fits = blk_any && (long long)slot < p.pool_blocks;
        if (lane == 0) {
            nzb[blk_id] = fits ? 1 : 0;
            if (fits) idxb[blk_id] = (int32_t)slot;
            if (blk_any && !fits) p.hdr->pool_overflow = 1;
        }
        if (!fits) return;
        // the whole 32 x 32 block, row-major (entries outside the grid are never read)
        float *dst = p.pool + (size_t)slot * (kBlk * kBlk);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            float v[4];
            read4(it, v);
            *reinterpret_cast<float4 *>(dst + ((lane >> 3) + 8 * it) * kBlk + c4) = make_float4(v[0], v[1], v[2], v[3]);
        }
        return;
    }
    if (lane == 0) nzb[blk_id] = blk_any ? 1 : 0;
    if (!blk_any) return;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        float v[4];
        read4(it, v);
        const int row = row0 + rb * 32 + (lane >> 3) + 8 * it;
        if (row < p.N) {
            float *q = Eb + (size_t)row * p.M + j0 + c4;
            if (p.vec_m && j0 + c4 + 3 < p.M) {
                *reinterpret_cast<float4 *>(q) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j0 + c4 + e < p.M) q[e] = v[e];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Input gradients where E is produced (Sec. 4.3, last two equations):
//   dx_i = 2 (x_i sum_j E_ij - sum_j E_ij y_j),     dy_j = 2 (y_j sum_i E_ij - sum_i E_ij x_i).
// One wavefront contracts a finished 32x32 block of E (in the ring, skewed) against the 32 rows of y
// and of x it meets, on the fp16 matrix cores with both operands split into two float16 pieces
// (E * 2^10; the sequence rows times one power-of-two scale per block, the largest of the rows'
// scales, from the per-row scales the forward call stored): a1*b1 + a1*b2 + a2*b1, float32
// accumulate, the same arithmetic as input_grad_half_kernel.  gradient_finish_kernel applies the
// rest of the formula afterwards.  A block whose entries are all below 2^-40 adds nothing (what that
// drops is below 2^-40 M max|y| per gradient entry) and is left after one look at its entries.
//
// Where the sums go.  Rows i0.. of the x side belong to this band alone: sum_j E_ij y_j and sum_j E_ij
// are added to p.gdx (the caller's dx) and p.rsum in float32, block after block in the order of the
// sweep.  Columns j0.. of the y side receive a term from every band of the pair, and the bands of a
// pair run at the same time: their terms are added with integer atomics to a fixed-point number per
// entry, so that the sum does not depend on who comes first (integer addition commutes exactly; a
// float32 atomic would not).  The number has unit 2^(e_b - prec), e_b = exponent bound of pair b's x
// (|x| < 2^e_b, p.pair_exp), and two 32-bit words: the low p.fx_lo_bits bits of every term are added
// to one word (p.gdy, the caller's dy, as unsigned), the rest to the other (p.gdy_hi); neither can
// overflow with as many terms as the pair has blocks in a column (the host chooses the widths).
// ---------------------------------------------------------------------------------------------
constexpr float kGradLive = 9.094947e-13f;  // 2^-40
constexpr int kMargBits = 24;               // fixed-point digits of the column sums of E (terms <= 33)

__device__ __forceinline__ void fixed_point_add(unsigned *lo_word, int *hi_word, float v, int shift, int lo_bits)
{
    const long long q = __float2ll_rn(ldexpf(v, shift));
    const unsigned lo = (unsigned)(q & ((1ll << lo_bits) - 1));
    const int hi = (int)(q >> lo_bits);
    if (lo != 0u) atomicAdd(lo_word, lo);
    if (hi != 0) atomicAdd(hi_word, hi);
}

template <int NFT, int COLS = kRingCols, int STRIDE = kRingStride>
__device__ __attribute__((noinline)) void grad_E_block(const Params &p, SweepRange rg, const float *ring, int rb, int cb,
                                                       int row0, int b, int Nl, int Ml, int lane)
{
    if (cb < 0 || cb >= p.ncb || row0 + 32 * rb >= p.N || !block_in_range(rg, rb, cb)) return;
    const int r = lane & 31, h = lane >> 5;
    const int i0 = row0 + 32 * rb, j0 = cb * kBlk;
    const int sb = 32 * (cb + rb);  // step at which band row 32*rb meets column j0
    // E[i0 + r][j0 + 16 ks + 8 h + c]: the A operand of the product with y, and every entry of the
    // block once over the wavefront
    float ea[2][8];
    {
        const float *rowp = ring + (32 * rb + r) * STRIDE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                // (ring positions of cells beyond the pair's grid may belong to macro-steps that never ran)
                const float v = rowp[(sb + r + 16 * ks + 8 * h + c) & (COLS - 1)];
                ea[ks][c] = (i0 + r < Nl && j0 + 16 * ks + 8 * h + c < Ml) ? v : 0.f;
            }
    }
    bool any = false;
    float rs = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            any |= ea[ks][c] >= kGradLive;
            rs += ea[ks][c];
        }
    if (!__any(any)) return;
    rs += __shfl_xor(rs, 32);
    if (h == 0 && i0 + r < p.N) p.rsum[(size_t)b * p.N + i0 + r] += rs;

    const float sA = 1024.0f;
    if (p.gdx != nullptr) {
        const unsigned *yis = reinterpret_cast<const unsigned *>(p.yis + b * p.yn_stride);
        // (positive powers of two: their bit patterns order like the values)
        const float ismax = wave_max_f32(__uint_as_float(yis[min(j0 + r, Ml - 1)]));
        const float sB = 1.0f / ismax, unscale = ismax * (1.0f / 1024.0f);
        half8 a1[2], a2[2];
        split8(ea[0], sA, a1[0], a2[0]);
        split8(ea[1], sA, a1[1], a2[1]);
        const float *yb = p.y + b * p.y_stride;
        float *g = p.gdx + ((size_t)b * p.N + i0) * p.D;
        // all operand values and all sums so far are asked for before the first is used
        float bv[NFT][2][8], old[NFT][16];
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            const int f = 32 * t + r;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int jb = j0 + 16 * ks + 8 * h;
                const float *src = yb + (size_t)jb * p.D + f;
#pragma unroll
                for (int c = 0; c < 8; ++c) bv[t][ks][c] = (jb + c < Ml && f < p.D) ? src[(size_t)c * p.D] : 0.f;
            }
        }
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            const int f = 32 * t + r;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int rr = 8 * (q >> 2) + 4 * h + (q & 3);
                old[t][q] = (i0 + rr < p.N && f < p.D) ? g[(size_t)rr * p.D + f] : 0.f;
            }
        }
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            const int f = 32 * t + r;
            floatx16 acc = zero16();
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                half8 b1, b2;
                split8(bv[t][ks], sB, b1, b2);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[ks], b1, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[ks], b2, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2[ks], b1, acc, 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int rr = 8 * (q >> 2) + 4 * h + (q & 3);
                if (i0 + rr < p.N && f < p.D) g[(size_t)rr * p.D + f] = fmaf(acc[q], unscale, old[t][q]);
            }
        }
    }
    if (p.gdy != nullptr) {
        // E[i0 + 16 ks + 8 h + c][j0 + r]: the A operand of the product with x
        float et[2][8];
        float cs = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int rr = 16 * ks + 8 * h + c;
                const float v = ring[(32 * rb + rr) * STRIDE + ((sb + r + rr) & (COLS - 1))];
                et[ks][c] = (i0 + rr < Nl && j0 + r < Ml) ? v : 0.f;
                cs += et[ks][c];
            }
        cs += __shfl_xor(cs, 32);
        if (h == 0 && j0 + r < p.M)
            fixed_point_add(p.csum_lo + (size_t)b * p.M + j0 + r, p.csum_hi + (size_t)b * p.M + j0 + r, cs, kMargBits, p.fx_lo_bits);
        const unsigned *xis = reinterpret_cast<const unsigned *>(p.xis + b * p.xn_stride);
        const float ismax = wave_max_f32(__uint_as_float(xis[min(i0 + r, Nl - 1)]));
        const float sB = 1.0f / ismax, unscale = ismax * (1.0f / 1024.0f);
        half8 a1[2], a2[2];
        split8(et[0], sA, a1[0], a2[0]);
        split8(et[1], sA, a1[1], a2[1]);
        const float *xb = p.x + b * p.x_stride;
        const int shift = p.fx_prec - p.pair_exp[b];
        unsigned *glo = reinterpret_cast<unsigned *>(p.gdy) + ((size_t)b * p.M + j0) * p.D;
        int *ghi = p.gdy_hi + ((size_t)b * p.M + j0) * p.D;
        float bv[NFT][2][8];
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            const int f = 32 * t + r;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int ib = i0 + 16 * ks + 8 * h;
                const float *src = xb + (size_t)ib * p.D + f;
#pragma unroll
                for (int c = 0; c < 8; ++c) bv[t][ks][c] = (ib + c < Nl && f < p.D) ? src[(size_t)c * p.D] : 0.f;
            }
        }
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            const int f = 32 * t + r;
            floatx16 acc = zero16();
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                half8 b1, b2;
                split8(bv[t][ks], sB, b1, b2);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[ks], b1, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[ks], b2, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2[ks], b1, acc, 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int cc = 8 * (q >> 2) + 4 * h + (q & 3);
                if (j0 + cc < p.M && f < p.D)
                    fixed_point_add(glo + (size_t)cc * p.D + f, ghi + (size_t)cc * p.D + f, acc[q] * unscale, shift, p.fx_lo_bits);
            }
        }
    }
}

// the same for any D <= 128: 32 features per pass of the matrix cores
__device__ __forceinline__ void grad_E_block_any(const Params &p, const SweepRange &rg, const float *ring, int rb, int cb,
                                                 int row0, int b, int Nl, int Ml, int lane)
{
    if (p.D <= 32)
        grad_E_block<1>(p, rg, ring, rb, cb, row0, b, Nl, Ml, lane);
    else if (p.D <= 64)
        grad_E_block<2>(p, rg, ring, rb, cb, row0, b, Nl, Ml, lane);
    else
        grad_E_block<4>(p, rg, ring, rb, cb, row0, b, Nl, Ml, lane);
}

template <int KCH, int SLOTS, int NPROD, bool GRAD = false>
__device__ __forceinline__ void reverse_dp_body(const Params &p, WgShared<SLOTS> &sh, unsigned &ticket_s,
                                                double (&edge_out)[SLOTS][kEdgeOut], double (&hand)[kHandDoubles])
{
    static_assert(SLOTS == 4 || SLOTS == 2 || SLOTS == 1, "supported workgroup shapes");
    static_assert(NPROD == 1 || (NPROD == 2 && KCH > 0), "two producers only split MFMA work");
    constexpr int kThreads = wg_threads(SLOTS, NPROD);
    // One band or a chained pair per workgroup are the shapes of small problems, where this sweep
    // runs beside the forward sweep: it cannot use R, so it only stores its own table for
    // alignment_kernel.
    constexpr bool TSWEEP = (SLOTS == 1 || SLOTS == 2);
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (p.hdr->abort_backward) return;
    if constexpr (GRAD) {
        if (p.hdr->pool_overflow == 0) return;  // the pool held every block: the gradients are done
    }

    if (threadIdx.x == 0) ticket_s = atomicAdd(&p.hdr->bwd_ticket, 1u);
    for (int e = threadIdx.x; e < SLOTS * kRingFloats; e += kThreads) (&sh.ring[0][0])[e] = kBigCost;
    int producer, slot;  // producer: 0 = consumer, 1.. = producer number
    if constexpr (SLOTS == 4) {
        elect_role(sh, lane, w, 1 + NPROD, producer, slot);
    } else if constexpr (SLOTS == 2) {
        for (int e = threadIdx.x; e < kHandDoubles; e += kThreads) hand[e] = kBig;
        chain_role(w, producer, slot);
        __syncthreads();
    } else {
        producer = w;
        slot = 0;
        __syncthreads();
    }
    const unsigned ticket = __builtin_amdgcn_readfirstlane(ticket_s);
    int kk, b;  // kk counts bands from the last one
    SweepRange rg;  // macro-steps to run, from the ticket alone (the same for every wavefront of the workgroup)
    if constexpr (SLOTS == 2) {
        const int kp = ticket / (unsigned)p.B;
        b = ticket - kp * p.B;
        kk = 2 * kp + (slot & 1);
        const int k_low = p.nbands - 1 - 2 * kp;  // the lower band of the pair (slot 0), the upper one is k_low - 1
        rg = sweep_range(p, max(k_low - 1, 0) * kBandRows, k_low * kBandRows, pair_len(p.x_len, b, p.N),
                         pair_len(p.y_len, b, p.M));
    } else {
        const int ngroups = (p.B + SLOTS - 1) / SLOTS;
        kk = ticket / (unsigned)ngroups;
        const int b0 = (ticket - kk * ngroups) * SLOTS;
        b = b0 + slot;
        int nl = 1, ml = 1;  // the longest sequences among the workgroup's pairs
        for (int s2 = 0; s2 < SLOTS; ++s2) {
            if (b0 + s2 < p.B) {
                nl = max(nl, pair_len(p.x_len, b0 + s2, p.N));
                ml = max(ml, pair_len(p.y_len, b0 + s2, p.M));
            }
        }
        rg = sweep_range(p, (p.nbands - 1 - kk) * kBandRows, (p.nbands - 1 - kk) * kBandRows, nl, ml);
    }
    const int k = p.nbands - 1 - kk;
    const bool live = (kk < p.nbands) && (b < p.B) && rg.hi >= rg.lo;
    const int lag = (SLOTS == 2) ? kChainLag * slot : 0;
    const int niter = max(rg.hi - rg.lo + 1, 0) + ((SLOTS == 2) ? kChainLag : 0);
    if constexpr (SLOTS == 2) {
        if (producer < 0) {  // unused wavefront: only keeps the barrier count (one before the loop, one per iteration)
            for (int it = 0; it <= niter; ++it) __syncthreads();
            return;
        }
    }

    const int M = p.M, N = p.N;
    const int row0 = (live ? k : 0) * kBandRows;
    float *ring = sh.ring[slot];
    const int bb = live ? b : 0;
    const int Nl = pair_len(p.x_len, bb, N), Ml = pair_len(p.y_len, bb, M);  // the pair's own lengths
    Params pl = p;
    pl.N = Nl;
    pl.M = Ml;
    [[maybe_unused]] const float *xb = p.x + bb * p.x_stride, *yb = p.y + bb * p.y_stride;
    const float *xnb = p.xn + bb * p.xn_stride, *ynb = p.yn + bb * p.yn_stride;
    const float *xisb = p.xis + bb * p.xn_stride, *yisb = p.yis + bb * p.yn_stride;
    const uint16_t *xh = p.xh + bb * p.xh_stride, *yh = p.yh + bb * p.yh_stride;
    float2 *rowtab = sh.rowtab[slot];
    const int sg0 = rg.hi;  // the sweep's first macro-step

    float *Eb = p.E + (size_t)bb * N * M;
    unsigned char *nzb = p.nz + (size_t)bb * p.nrb * p.ncb;
    int32_t *idxb = p.idx != nullptr ? p.idx + (size_t)bb * p.nrb * p.ncb : nullptr;  // compact E
    // Who writes the finished E blocks out: the producer, whose loads and stores then wait beside the
    // consumer's chain instead of in it (measured with recomputation at the L = 8192 shape: 6.3 -> 5.3 ms
    // at D = 16, 6.5 -> 6.1 ms at D = 64) - except where the producer has no registers left for it
    // (recomputation with D > 64: the x pieces fill them, the flush would spill).
    // GRAD: E is not written out at all; the consumer contracts each finished block into the gradients
    // (grad_E_block) right after it has published the macro-step's boundary values.
    static_assert(!GRAD || dp_recompute(KCH, SLOTS), "the contracting sweep is the recomputing one");
    constexpr bool kProducerFlush = !GRAD && !TSWEEP && !(dp_recompute(KCH, SLOTS) && KCH > 4);

    if (producer) {
        // Besides the cost blocks, the producers write out the E blocks the consumer finished in the
        // previous macro-step `done`: (upper rows, done) and (lower rows, done-1).  Each producer
        // touches only the rows it owns and flushes before it overwrites the same ring phase.
        auto flush = [&](int done, bool upper, bool lower) {
            if constexpr (kProducerFlush) {
                const bool dead = sh.blk_dead[slot][done & 1] != 0;  // written by the consumer before the last barrier
                if (upper) flush_E_block(p, rg, ring, Eb, nzb, 0, done, row0, lane, dead, 0, idxb);
                if (lower) flush_E_block(p, rg, ring, Eb, nzb, 1, done - 1, row0, lane, dead, 0, idxb);
            }
        };
        // blocks the first macro-step reads: (upper rows, sg0-1), (lower rows, sg0-1), (lower rows, sg0-2)
        if constexpr (KCH > 0 && NPROD == 2) {
            // producer 1 makes (upper rows, sg-2), producer 2 makes (lower rows, sg-3)
            auto body = [&](auto &mp, bool upper) {
                if (live) {
                    mp.init(pl, xh, xnb, xisb, rowtab, row0, lane);
                    if (upper) {
                        mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 0, sg0 - 1, row0, lane);
                    } else {
                        mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 1, sg0 - 1, row0, lane);
                        mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 1, sg0 - 2, row0, lane);
                    }
                    mp.prime(pl, yh, ynb, yisb, sg0, lane);
                }
                __syncthreads();
                for (int it = 0; it < niter; ++it) {
                    const int sg = sg0 - (it - lag);
                    if (live && sg >= rg.lo && sg <= sg0) {
                        if (sg < sg0) flush(sg + 1, upper, !upper);
                        mp.run(pl, yh, ynb, yisb, ring, rowtab, sg, row0, lane);
                    }
                    __syncthreads();
                }
                if (live) flush(rg.lo, upper, !upper);
            };
            if (producer == 1) {
                HalfProducer<KCH, -1, 0, 1> mp;
                body(mp, true);
            } else {
                HalfProducer<KCH, -1, 1, 1> mp;
                body(mp, false);
            }
        } else if constexpr (KCH > 0) {
            HalfProducer<KCH, -1, 0, 2> mp;
            if (live) {
                mp.init(pl, xh, xnb, xisb, rowtab, row0, lane);
                mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 0, sg0 - 1, row0, lane);
                mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 1, sg0 - 1, row0, lane);
                mp.block_now(pl, yh, ynb, yisb, ring, rowtab, 1, sg0 - 2, row0, lane);
                mp.prime(pl, yh, ynb, yisb, sg0, lane);
            }
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = sg0 - (it - lag);
                if (live && sg >= rg.lo && sg <= sg0) {
                    if (sg < sg0) flush(sg + 1, true, true);
                    mp.run(pl, yh, ynb, yisb, ring, rowtab, sg, row0, lane);
                }
                __syncthreads();
            }
            if (live) flush(rg.lo, true, true);
        } else if constexpr (KCH == 0) {
            if (live) {
                generic_block(pl, b, ring, 0, sg0 - 1, row0, lane);
                generic_block(pl, b, ring, 1, sg0 - 1, row0, lane);
                generic_block(pl, b, ring, 1, sg0 - 2, row0, lane);
            }
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = sg0 - (it - lag);
                if (live && sg >= rg.lo && sg <= sg0) {
                    if (sg < sg0) flush(sg + 1, true, true);
                    generic_block(pl, b, ring, 0, sg - 2, row0, lane);
                    generic_block(pl, b, ring, 1, sg - 3, row0, lane);
                }
                __syncthreads();
            }
            if (live) flush(rg.lo, true, true);
        } else {
            const float *cost_b = p.cost + (size_t)bb * N * M;
            float4 pre[2][4];
            if (live) {
                load_cost_block(pre[0], cost_b, 0, sg0 - 1, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                store_cost_block(ring, pre[0], 0, sg0 - 1, lane);
                load_cost_block(pre[0], cost_b, 1, sg0 - 1, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                store_cost_block(ring, pre[0], 1, sg0 - 1, lane);
                load_cost_block(pre[0], cost_b, 1, sg0 - 2, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                store_cost_block(ring, pre[0], 1, sg0 - 2, lane);
                load_cost_block(pre[0], cost_b, 0, sg0 - 2, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                load_cost_block(pre[1], cost_b, 1, sg0 - 3, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
            }
            __syncthreads();
            for (int it = 0; it < niter; ++it) {
                const int sg = sg0 - (it - lag);
                if (live && sg >= rg.lo && sg <= sg0) {
                    if (sg < sg0) flush(sg + 1, true, true);
                    store_cost_block(ring, pre[0], 0, sg - 2, lane);
                    store_cost_block(ring, pre[1], 1, sg - 3, lane);
                    load_cost_block(pre[0], cost_b, 0, sg - 3, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                    load_cost_block(pre[1], cost_b, 1, sg - 4, row0, Nl, Ml, M, p.window, p.vec_m != 0, lane);
                }
                __syncthreads();
            }
            if (live) flush(rg.lo, true, true);
        }
        return;
    }

    // ---------------------------------------------------------------------- consumer wavefront
    // The chain of dependent steps is what everything waits for: where this wavefront shares its SIMD
    // with producers, its instructions go first.
    __builtin_amdgcn_s_setprio(3);
    // CH: -1 = both neighbouring bands are reached through memory; 0 = the band above is the other
    // band of this workgroup (this band's first row goes to the LDS hand-over ring); 1 = the band
    // below is.
    auto consume = [&](auto chain_c) {
    constexpr int CH = decltype(chain_c)::value;
    const double c2d = p.c2d;  // log2(e)/gamma
    bool gave_up = false;
    double right = kBig;  // T[i][j+1]
    double diag = kBig;   // T[i+1][j+1]
    // step at which this lane meets the cell whose diagonal successor is T[N+1,M+1] = 0, and the
    // macro-step in which that happens in this band
    const int s_corner = (live && row0 + lane == Nl - 1) ? (Ml - 1 + lane) : -1;
    const int t_last = Nl - 1 - row0;
    const int sg_corner = (live && t_last >= 0 && t_last < kBandRows) ? (Ml - 1 + t_last) / kBlk : -1;
    const double Rfin = (live && !TSWEEP) ? p.rfinal[b] : 0.0;
    const int kc = live ? k : 0;
    const bool has_below = live && (k + 1 < p.nbands) && CH != 1;  // through memory
    const bool emit_top = live && k > 0;                           // the band's first row goes to memory
    constexpr bool RECOMP = dp_recompute(KCH, SLOTS);
    static_assert(RECOMP != TSWEEP, "a reverse sweep either stores its own table or recomputes R and forms E");
    const unsigned long long *brow_in = p.brow_b + ((size_t)bb * p.nbands + (has_below ? kc + 1 : kc)) * M;
    unsigned long long *brow_out = p.brow_b + ((size_t)bb * p.nbands + kc) * M;
    // (table pointers are those of the band's macro-step 0; the table starts at macro-step table_base)
    const ptrdiff_t tb = table_base(p, kc);
    const ptrdiff_t band_off = (((ptrdiff_t)bb * p.nbands + kc) * (ptrdiff_t)p.nm_tab - tb) * kBlk * kBandRows;
    double *Qk = TSWEEP ? p.Q + band_off : nullptr;
    const double *Ck = RECOMP ? p.ckpt + (((ptrdiff_t)bb * p.nbands + kc) * (ptrdiff_t)p.nm_tab - tb) * 2 * kBandRows : nullptr;
    // the forward's row above this band (final values, written by the forward call)
    const double *ftop_g = reinterpret_cast<const double *>(p.brow) + ((size_t)bb * p.nbands + (kc > 0 ? kc - 1 : 0)) * M;
    double *ftop = sh.ftop[slot];
    float *my_ring = ring + lane * kRingStride;
    double *bot = sh.edge_in[slot];
    double *eo = edge_out[slot];

    bool dead_prev = true;  // the macro-step before the first one: beyond the table, nothing there
    // R of the first macro-step; afterwards each value is reloaded one macro-step ahead, right after use
    double Rq[kBlk];
    double ck_left = kBig, ck_diag = kBig;  // RECOMP: forward lane state at the start of the coming macro-step
    double ftop_next = kBig;                // RECOMP: forward's row above the band for the coming macro-step
    if constexpr (RECOMP) {
        if (live) {
            ck_left = Ck[((size_t)sg0 * 2 + 0) * kBandRows + lane];
            ck_diag = Ck[((size_t)sg0 * 2 + 1) * kBandRows + lane];
            const int jf = sg0 * kBlk + lane;
            if (k > 0 && lane < kBlk && jf < M) ftop_next = ftop_g[jf];
        }
    }

    // row below the band for the first macro-step: lane l >= 32 brings column 32*sg - 63 + (l - 32),
    // which lane 63 meets at step u = l - 32
    if constexpr (CH != 1) {
        double b0 = kBig;
        if (has_below) {
            const int jj = sg0 * kBlk + lane - kBlk - (kBandRows - 1);
            const bool need = lane >= kBlk && jj >= 0 && jj < M;
            b0 = resolve_boundary(p, brow_in, jj, need, lane, gave_up, peek_boundary(brow_in, jj, need));
        }
        if (lane >= kBlk) bot[lane - kBlk] = b0;
    }
    __syncthreads();

    for (int it = 0; it < niter; ++it) {
        const int sg = sg0 - (it - lag);
        if (live && sg >= rg.lo && sg <= sg0) {
            unsigned long long nxt_bits = (unsigned long long)__double_as_longlong(kBig);
            const int jn = (sg - 1) * kBlk + lane - kBlk - (kBandRows - 1);
            const bool need_n = has_below && lane >= kBlk && jn >= 0 && jn < M;
            float *rd = my_ring + (sg & 3) * kBlk;
            // The row below, column 32*sg + u - 63 at step u: from the incoming boundary values, or
            // from the hand-over ring, where the band below put column c at slot c mod 128.
            const double *bot31 = bot + (kBlk - 1), *bot0 = bot;  // step 31, steps 0..30
            if constexpr (CH == 1) {
                bot31 = hand + ((sg - 1) & 3) * kBlk;
                bot0 = hand + ((sg - 2) & 3) * kBlk + 1;
            }
            // lane 0's values are the band's first row (column 32*sg + u at step u)
            double *my_eo = eo + ((lane == 0) ? 0 : kBlk + lane);
            if constexpr (CH == 0) my_eo = hand + ((lane == 0) ? (sg & 3) * kBlk : kHandRing + lane);
            double *Qs = TSWEEP ? Qk + (size_t)sg * kBlk * kBandRows : nullptr;
            const int sbase = sg * kBlk;
            // Can any cell of this macro-step have a non-zero E (in float32)?  Every R of the macro-step
            // is at least the smallest value entering it (the lanes' forward state at its start, the
            // row above) minus 32 log2(3), since a cell is its non-negative cost plus a soft-minimum
            // of its predecessors; likewise every Q = T - d and the reverse state (the lanes' values,
            // the row below).  If R[N,M] - min R - min Q is far below the smallest float32 exponent,
            // E is zero throughout: the macro-step only continues T (no recomputation, no exp2).
            bool dead = false;
            if constexpr (RECOMP) {
                float rmin = (float)min_f64(ck_left, ck_diag), qmin = (float)min_f64(right, diag);
                if (lane < kBlk) {
                    rmin = fminf(rmin, (float)ftop_next);
                    qmin = fminf(qmin, (float)bot[lane]);
                }
                rmin = wave_min_f32(rmin);
                qmin = wave_min_f32(qmin);
                // 157 (float32), 2 x 32 log2(3) = 102, rounding of the two minima to float32 (<= 2 x 16)
                dead = __builtin_amdgcn_readfirstlane((int)(((double)rmin + (double)qmin > Rfin + 300.0) && sg != sg_corner)) != 0;
            }
            if constexpr (RECOMP) {
                // recompute R of this macro-step from the forward's checkpoint (same arithmetic, same
                // cost values, hence the same bits the forward had)
                double fl = ck_left, fd = ck_diag;
                if (lane < kBlk) ftop[lane] = ftop_next;
                if (sg > rg.lo) {  // everything the next macro-step's recomputation needs, one macro-step ahead
                    ck_left = __builtin_nontemporal_load(&Ck[((size_t)(sg - 1) * 2 + 0) * kBandRows + lane]);
                    ck_diag = __builtin_nontemporal_load(&Ck[((size_t)(sg - 1) * 2 + 1) * kBandRows + lane]);
                    const int jf = sbase - kBlk + lane;
                    ftop_next = kBig;
                    if (k > 0 && lane < kBlk && jf < M) ftop_next = __builtin_nontemporal_load(&ftop_g[jf]);
                }
                if (!dead) {
#pragma unroll
                    for (int u = 0; u < kBlk; ++u) {
                        const double up = lane_shr1(fl, ftop[u]);
                        const float dcf = rd[u];
                        double mf;
                        float Lf;
                        softmin3_parts(fd, up, fl, mf, Lf);
                        const double cur = fma((double)dcf, c2d, mf) - (double)Lf;
                        Rq[u] = Rfin - cur;
                        fd = up;
                        fl = cur;
                    }
                }
            }
            // (small problems: the macro-step's 32 cost values in one batch, as in the forward sweep)
            [[maybe_unused]] float dcv[TSWEEP ? kBlk : 1];
            if constexpr (TSWEEP) {
#pragma unroll
                for (int u = 0; u < kBlk; ++u) dcv[u] = rd[u];
            }
            auto steps = [&](auto corner, auto alive) {
#pragma unroll
            for (int u = kBlk - 1; u >= 0; --u) {
                if (u == kBlk - 1 - kPeekStep && has_below) nxt_bits = peek_boundary(brow_in, jn, need_n);
                const double down = lane_shl1(right, u == kBlk - 1 ? bot31[0] : bot0[u]);  // T[i+1][j]; lane 63 takes the row below the band
                float dc;
                if constexpr (TSWEEP)
                    dc = dcv[u];
                else
                    dc = rd[u];
                const double dg = (decltype(corner)::value && sbase + u == s_corner) ? 0.0 : diag;
                double m;
                float L;
                softmin3_parts(dg, down, right, m, L);
                double cur;
                if constexpr (TSWEEP) {
                    // the soft-minimum part Q = T - d goes to the table: log2 E = R[N,M] - R[i,j] - Q[i,j]
                    const double q = m - (double)L;
                    __builtin_nontemporal_store(q, &Qs[u * kBandRows + lane]);
                    cur = fma((double)dc, c2d, q);
                } else {
                    cur = fma((double)dc, c2d, m) - (double)L;
                    if constexpr (decltype(alive)::value) {
                        // log2 E = R[N,M] - R[i,j] - (m - L) in table units
                        rd[u] = __builtin_amdgcn_exp2f((float)(Rq[u] - m) + L);
                    } else {
                        rd[u] = 0.0f;
                    }
                }
                my_eo[u] = cur;  // lane 0: value of column 32*sg + u for the band above
                diag = down;
                right = cur;
            }
            };
            if (sg == sg_corner)
                steps(std::true_type{}, std::true_type{});
            else if (RECOMP && dead)
                steps(std::false_type{}, std::false_type{});
            else
                steps(std::false_type{}, std::true_type{});
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            // first row of the band, columns 32*sg .. 32*sg+31, for the band above
            if (emit_top && lane < kBlk) {
                const int j = sg * kBlk + lane;
                // (also from a chained pair's lower band, whose first row travels through LDS: see the forward sweep)
                const double *src = (CH == 0) ? hand + (sg & 3) * kBlk : eo;
                if (j < M) publish_boundary(brow_out, j, src[lane]);
            }
            // the E blocks this macro-step completed, (upper rows, sg) and (lower rows, sg-1): written
            // out by the producers during the next macro-step, or here
            // (both hold cells of this macro-step and the one before it only)
            const bool blocks_dead = dead && dead_prev;
            dead_prev = dead;
            if constexpr (GRAD) {
                // into the gradients, once the band above has what it waits for
                // (the routine is out of line and takes the parameters by reference: from the copy in the
                // workspace, or the kernel would have to hold one in scratch memory)
                if (!blocks_dead) {
                    grad_E_block_any(*p.self, rg, ring, 0, sg, row0, bb, Nl, Ml, lane);
                    grad_E_block_any(*p.self, rg, ring, 1, sg - 1, row0, bb, Nl, Ml, lane);
                }
            } else if constexpr (!kProducerFlush && !TSWEEP) {
                flush_E_block(p, rg, ring, Eb, nzb, 0, sg, row0, lane, blocks_dead, 0, idxb);
                flush_E_block(p, rg, ring, Eb, nzb, 1, sg - 1, row0, lane, blocks_dead, 0, idxb);
            } else if constexpr (!TSWEEP) {
                if (lane == 0) sh.blk_dead[slot][sg & 1] = blocks_dead ? 1 : 0;
            }
            if constexpr (CH != 1) {
                double bn = kBig;
                if (has_below) bn = resolve_boundary(p, brow_in, jn, need_n, lane, gave_up, nxt_bits);
                if (lane >= kBlk) bot[lane - kBlk] = bn;
            }
        }
        __syncthreads();
    }
    };
    if constexpr (SLOTS == 2) {
        if (slot == 0)
            consume(std::integral_constant<int, 0>{});
        else
            consume(std::integral_constant<int, 1>{});
    } else {
        consume(std::integral_constant<int, -1>{});
    }
}

// ---------------------------------------------------------------------------------------------
// Alignment matrix from the two tables (small problems, where the forward call ran both sweeps).
// With T the reverse DP over the same costs, R[i,j] + T[i,j] - d[i,j] is the soft-minimum cost of
// all alignments through cell (i,j), so
//     E[i,j] = exp((R[N,M] - R[i,j] - T[i,j] + d[i,j]) / gamma),
// which satisfies the log-space recurrence of Sec. 4.2 (divide that recurrence by E and substitute).
// The reverse sweep stores Q = T - d (its soft-minimum part), so no cost is needed here, and both
// tables are in units of gamma*ln2:  log2 E = R[N,M] - R - Q.
// One wavefront (a workgroup of its own, no barriers) streams a run of `seg_blocks` 32-column
// blocks of one band: per macro-step it reads the 32 step-rows of both tables (512 contiguous
// bytes each, the next macro-step's already in flight), puts E into its LDS ring exactly as the
// reverse-sweep consumer of the large problems does, and writes out the two 32x32 blocks that
// became complete, row-major, with their "any non-zero" flags.  Both blocks only hold cells of
// the last two macro-steps, so the ring has two phases of 32 steps.  Only the two macro-steps
// past a run's end are read twice.
// ---------------------------------------------------------------------------------------------
constexpr int kAlignRingCols = 64, kAlignRingStride = 65;

// Which columns of band k can hold a non-zero E (in float32)?  Every alignment path through a cell
// (i,j) of the band enters the band at a column <= j and leaves it at a column >= j, so
//   E[i,j] <= P(enter at a column <= j)  and  E[i,j] <= P(leave at a column >= j).
// Both probabilities follow from the boundary rows the two sweeps left behind: the path's first
// cell in row r+1 is (r+1,j) with probability
//   2^(R[N,M] - T[r+1,j] - softmin2(R[r,j], R[r,j-1]))          (r = the last row of the band above),
// and its last cell in row r is (r,j) with probability
//   2^(R[N,M] - R[r,j] - softmin2(T[r+1,j], T[r+1,j+1]))        (r = the band's own last row),
// in table units, softmin2 >= min - 1.  With thr = -(156 + log2 M) every column left of the first one
// whose entering term exceeds thr has E < M * 2^thr, which float32 cannot tell from 0, and likewise
// right of the last column whose leaving term exceeds thr.  Returns that column range (the whole row
// for the first band's left end and for the right end of the band that holds the pair's last row).
__device__ __forceinline__ void live_columns(const Params &p, int b, int k, int Nl, int Ml, double Rfin, int lane,
                                             int &first, int &last)
{
    const double thr = -(157.0 + (double)(32 - __builtin_clz((unsigned)p.M)));
    auto row = [&](const unsigned long long *rows, int band, int j) {
        return __longlong_as_double((long long)rows[((size_t)b * p.nbands + band) * p.M + j]);
    };
    // under a band constraint only the columns within the window of the band's rows can matter
    const int row0 = k * kBandRows;
    const int jlo = p.window < kNoWindow ? max(0, row0 - p.window - 1) : 0;
    const int jhi = p.window < kNoWindow ? min(Ml - 1, row0 + kBandRows + p.window) : Ml - 1;
    // (kScan iterations' loads are asked for together: one memory round trip per 64*kScan columns, not per 64)
    constexpr int kScan = 8;
    first = jlo;
    if (k > 0) {
        int f = Ml;
        for (int j0 = jlo + lane; j0 <= jhi; j0 += kBandRows * kScan) {
            double ra[kScan], rb[kScan], tq[kScan];
#pragma unroll
            for (int i = 0; i < kScan; ++i) {
                const int j = j0 + i * kBandRows;
                const bool in = j <= jhi;
                ra[i] = in ? row(p.brow, k - 1, j) : kBig;
                rb[i] = (in && j > 0) ? row(p.brow, k - 1, j - 1) : kBig;
                tq[i] = in ? row(p.brow_b, k, j) : kBig;
            }
#pragma unroll
            for (int i = 0; i < kScan; ++i) {
                const int j = j0 + i * kBandRows;
                const double term = (Rfin - tq[i]) - min_f64(ra[i], rb[i]) + 1.0;
                if (j <= jhi && term > thr) f = min(f, j);
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) f = min(f, __shfl_xor(f, o));
        first = f;
    }
    last = jhi;
    if (k != (Nl - 1) / kBandRows && k + 1 < p.nbands) {
        int l = -1;
        for (int j0 = jlo + lane; j0 <= jhi; j0 += kBandRows * kScan) {
            double ta[kScan], tb[kScan], rq[kScan];
#pragma unroll
            for (int i = 0; i < kScan; ++i) {
                const int j = j0 + i * kBandRows;
                const bool in = j <= jhi;
                ta[i] = in ? row(p.brow_b, k + 1, j) : kBig;
                tb[i] = (in && j + 1 < Ml) ? row(p.brow_b, k + 1, j + 1) : kBig;
                rq[i] = in ? row(p.brow, k, j) : kBig;
            }
#pragma unroll
            for (int i = 0; i < kScan; ++i) {
                const int j = j0 + i * kBandRows;
                const double term = (Rfin - rq[i]) - min_f64(ta[i], tb[i]) + 1.0;
                if (j <= jhi && term > thr) l = max(l, j);
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) l = max(l, __shfl_xor(l, o));
        last = l;
    }
}

template <bool LOOK_FIRST>  // find the columns that can hold a non-zero E before reading the tables
__global__ __launch_bounds__(64) void alignment_kernel(Params p, int seg_blocks)
{
    __shared__ float ring[kBandRows * kAlignRingStride];
    const int lane = threadIdx.x;
    const int k = blockIdx.y, b = blockIdx.z;
    const int cb0 = blockIdx.x * seg_blocks, cb1 = min(cb0 + seg_blocks, p.ncb);
    const int row0 = k * kBandRows;

    if (backward_refused(p)) {
        // record why (the status word keeps a time-out of the sweeps), leave NaN to the later kernels
        if (lane == 0 && blockIdx.x == 0 && k == 0 && b == 0 && p.hdr->status == 0) {
            p.hdr->magic = kMagic;
            p.hdr->status = kStatusState;
            p.hdr->abort_backward = 1;
        }
        return;
    }

    float *Eb = p.E + (size_t)b * p.N * p.M;
    unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;
    const ptrdiff_t band_off = (((ptrdiff_t)b * p.nbands + k) * (ptrdiff_t)p.nm_tab - table_base(p, k)) * kBlk * kBandRows;
    const double *Rk = p.R + band_off, *Qk = p.Q + band_off;
    const double Rfin = p.rfinal[b];
    float *my_ring = ring + lane * kAlignRingStride;
    // With a band constraint (or per-pair lengths) only macro-steps rg.lo .. rg.hi of the tables exist.
    // The blocks of the run that the sweeps did not cover are outside the window: flags cleared.
    const int Nl = pair_len(p.x_len, b, p.N), Ml = pair_len(p.y_len, b, p.M);
    SweepRange rg = sweep_range(p, row0, row0, Nl, Ml);
    // ... and of those, only the blocks between the first and the last column that can hold a
    // non-zero E are formed; the rest is zero without looking (most of the grid when gamma is small).
    // (Looking costs one pass over four boundary rows before the first table row can be asked for:
    // worth it from 16 column blocks on - 138 -> 40 us at N = M = 1024, B = 32 - not at 8.
    // The host asks for it from 16 column blocks on.)
    if constexpr (LOOK_FIRST) {
        if (rg.hi >= rg.lo) {
            int first, last;
            live_columns(p, b, k, Nl, Ml, Rfin, lane, first, last);
            first = __builtin_amdgcn_readfirstlane(first);  // the same in every lane: keep them scalar
            last = __builtin_amdgcn_readfirstlane(last);
            if (first <= last) {
                rg.lo = max(rg.lo, first / kBlk);
                rg.hi = min(rg.hi, last / kBlk + 2);
                rg.hi_u = min(rg.hi_u, last / kBlk + 2);
                rg.cb_last = min(rg.cb_last, last / kBlk);
            }
        }
    }
    if (LOOK_FIRST || p.window < kNoWindow || p.x_len != nullptr || p.y_len != nullptr) {
        for (int cb = cb0 + lane; cb < cb1; cb += kBandRows) {
            if (row0 < p.N && !block_in_range(rg, 0, cb)) nzb[(size_t)(row0 / kBlk) * p.ncb + cb] = 0;
            if (row0 + kBlk < p.N && !block_in_range(rg, 1, cb)) nzb[(size_t)(row0 / kBlk + 1) * p.ncb + cb] = 0;
        }
    }
    const int g_first = max(cb0, rg.lo);
    const int g_end = min(min(cb1 + 2, p.nmacro), rg.hi + 1);  // macro-steps [g_first, g_end) hold every cell of the run
    if (g_first >= g_end) return;

    auto load = [&](int g, double (&r)[kBlk], double (&q)[kBlk]) {
        const size_t o = (size_t)g * kBlk * kBandRows + lane;
#pragma unroll
        for (int u = 0; u < kBlk; ++u) {
            r[u] = __builtin_nontemporal_load(&Rk[o + (size_t)u * kBandRows]);
            q[u] = __builtin_nontemporal_load(&Qk[o + (size_t)u * kBandRows]);
        }
    };
    auto process = [&](int g, const double (&r)[kBlk], const double (&q)[kBlk]) {
        float *wr = my_ring + (g & 1) * kBlk;  // step s = 32g + u sits at ring slot s mod 64
#pragma unroll
        for (int u = 0; u < kBlk; ++u) wr[u] = __builtin_amdgcn_exp2f((float)((Rfin - r[u]) - q[u]));
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        // complete now: (upper rows, block g-1) and (lower rows, block g-2)
        if (g - 1 >= cb0 && g - 1 < cb1) flush_E_block<kAlignRingCols, kAlignRingStride>(p, rg, ring, Eb, nzb, 0, g - 1, row0, lane);
        if (g - 2 >= cb0 && g - 2 < cb1) flush_E_block<kAlignRingCols, kAlignRingStride>(p, rg, ring, Eb, nzb, 1, g - 2, row0, lane);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    };

    double ra[kBlk], qa[kBlk], rb[kBlk], qb[kBlk];
    int g = g_first;
    load(g, ra, qa);
    while (g < g_end) {
        if (g + 1 < g_end) load(g + 1, rb, qb);
        process(g, ra, qa);
        if (++g >= g_end) break;
        if (g + 1 < g_end) load(g + 1, ra, qa);
        process(g, rb, qb);
        ++g;
    }
    // blocks whose last macro-steps lie beyond the table (all their cells are already in the ring)
    for (; g < cb1 + 2; ++g) {
        if (g - 1 >= cb0 && g - 1 < cb1) flush_E_block<kAlignRingCols, kAlignRingStride>(p, rg, ring, Eb, nzb, 0, g - 1, row0, lane);
        if (g - 2 >= cb0 && g - 2 < cb1) flush_E_block<kAlignRingCols, kAlignRingStride>(p, rg, ring, Eb, nzb, 1, g - 2, row0, lane);
    }
}

// The same for short rows (at most NM - 2 column blocks): one workgroup of NW wavefronts per block
// row (32 rows: half a band).  The block row's E fits in LDS (32 rows x 32*NM steps), so every
// table entry is read exactly once - a wavefront takes a macro-step, its two half-waves alternate
// steps - and after one barrier the ncb blocks are written out, one per wavefront at a time.  (The
// run-per-wavefront kernel above re-reads two macro-steps per run, which at 8 column blocks and
// runs of 2 is 60 % more table traffic, and it has a quarter of the wavefronts in flight.)
constexpr int kAlignRowMacro = 12;  // macro-steps of E that alignment_row_kernel keeps (49 KB of LDS)
template <int NM, int NW>
__global__ __launch_bounds__(64 * NW) void alignment_row_kernel(Params p)
{
    constexpr int kStride = kBlk * NM + 1, kCols = 512;  // kCols: a power of two >= 32*NM, so no index ever wraps
    static_assert(kBlk * NM <= kCols, "the steps must fit below the wrap-around of flush_E_block");
    __shared__ float ring[kBlk * kStride + 2 * kBlk];  // the last block of a row is read up to step 32*NM + 30
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int rb = blockIdx.x, k = blockIdx.y, b = blockIdx.z;
    const int row0 = k * kBandRows;

    // (the header is asked for now and looked at once the first table rows have been asked for:
    // the kernel is a few memory round trips long, this keeps it from being one longer)
    const bool refused = backward_refused(p);
    if (row0 + kBlk * rb >= p.N) return;

    float *Eb = p.E + (size_t)b * p.N * p.M;
    unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;
    const ptrdiff_t band_off = (((ptrdiff_t)b * p.nbands + k) * (ptrdiff_t)p.nm_tab - table_base(p, k)) * kBlk * kBandRows;
    const double *Rk = p.R + band_off, *Qk = p.Q + band_off;
    const double Rfin = p.rfinal[b];
    const SweepRange rg = sweep_range(p, row0, row0, pair_len(p.x_len, b, p.N), pair_len(p.y_len, b, p.M));
    // this block row's cells lie in macro-steps rb ... ncb + rb
    const int g_begin = max(rg.lo, rb), g_end = min(min(rg.hi, p.ncb + rb) + 1, min(p.nmacro, NM));
    const int half = lane >> 5, r = lane & 31;
    float *my_ring = ring + r * kStride + half;
    auto load = [&](int g, double (&rr)[kBlk / 2], double (&qq)[kBlk / 2]) {
        const size_t o = ((size_t)g * kBlk + half) * kBandRows + kBlk * rb + r;
#pragma unroll
        for (int u = 0; u < kBlk / 2; ++u) {
            rr[u] = __builtin_nontemporal_load(&Rk[o + (size_t)(2 * u) * kBandRows]);
            qq[u] = __builtin_nontemporal_load(&Qk[o + (size_t)(2 * u) * kBandRows]);
        }
    };
    auto process = [&](int g, const double (&rr)[kBlk / 2], const double (&qq)[kBlk / 2]) {
        float *wr = my_ring + g * kBlk;  // step s = 32g + 2u + half sits at position s of the row
#pragma unroll
        for (int u = 0; u < kBlk / 2; ++u) wr[2 * u] = __builtin_amdgcn_exp2f((float)((Rfin - rr[u]) - qq[u]));
    };
    {
        double ra[kBlk / 2], qa[kBlk / 2], rc[kBlk / 2], qc[kBlk / 2];
        int g = g_begin + w;
        if (g < g_end) load(g, ra, qa);
        if (refused) {
            // record why (the status word keeps a time-out of the sweeps), leave NaN to the later kernels
            if (threadIdx.x == 0 && rb == 0 && k == 0 && b == 0 && p.hdr->status == 0) {
                p.hdr->magic = kMagic;
                p.hdr->status = kStatusState;
                p.hdr->abort_backward = 1;
            }
            return;
        }
        if (p.window < kNoWindow || p.x_len != nullptr || p.y_len != nullptr) {
            // blocks the sweeps did not cover are outside the window or the pair's lengths: flags cleared
            for (int cb = threadIdx.x; cb < p.ncb; cb += 64 * NW)
                if (!block_in_range(rg, rb, cb)) nzb[(size_t)(row0 / kBlk + rb) * p.ncb + cb] = 0;
        }
        // macro-steps of this block row that the sweeps left out hold no cell of the grid: zero
        for (int gz = rb + w; gz <= min(p.ncb + rb, NM - 1); gz += NW) {
            if (gz >= g_begin && gz < g_end) continue;
#pragma unroll
            for (int u = 0; u < kBlk / 2; ++u) my_ring[gz * kBlk + 2 * u] = 0.f;
        }
        while (g < g_end) {
            if (g + NW < g_end) load(g + NW, rc, qc);
            process(g, ra, qa);
            g += NW;
            if (g >= g_end) break;
            if (g + NW < g_end) load(g + NW, ra, qa);
            process(g, rc, qc);
            g += NW;
        }
    }
    __syncthreads();
    for (int cb = w; cb < p.ncb; cb += NW)
        flush_E_block<kCols, kStride>(p, rg, ring, Eb, nzb, rb, cb, row0, lane, false, kBlk * rb);
}

// ---------------------------------------------------------------------------------------------
// Kernels: the sweeps alone (large problems: forward call, then backward call), or both in one
// launch (small problems: even workgroups sweep forward, odd ones in reverse; the two sweeps
// share nothing but the cost).
// ---------------------------------------------------------------------------------------------
template <int KCH, int SLOTS, int NPROD>
__global__ __launch_bounds__(wg_threads(SLOTS, NPROD)) void forward_dp_kernel(Params p, float *__restrict__ value)
{
    __shared__ WgShared<SLOTS> sh;
    __shared__ unsigned ticket_s;
    __shared__ double edge_out[SLOTS][kEdgeOut];
    __shared__ double hand[kHandDoubles];
    forward_dp_body<KCH, SLOTS, NPROD>(p, value, sh, ticket_s, edge_out, hand);
}

template <int KCH, int SLOTS, int NPROD, bool GRAD = false>
__global__ __launch_bounds__(wg_threads(SLOTS, NPROD)) void backward_dp_kernel(Params p)
{
    __shared__ WgShared<SLOTS> sh;
    __shared__ unsigned ticket_s;
    __shared__ double edge_out[SLOTS][kEdgeOut];
    __shared__ double hand[kHandDoubles];
    reverse_dp_body<KCH, SLOTS, NPROD, GRAD>(p, sh, ticket_s, edge_out, hand);
}

template <int KCH, int SLOTS, int NPROD>
__global__ __launch_bounds__(wg_threads(SLOTS, NPROD)) void both_sweeps_kernel(Params p, float *__restrict__ value)
{
    static_assert(SLOTS == 1 || SLOTS == 2, "the shapes of small problems");
    __shared__ WgShared<SLOTS> sh;
    __shared__ unsigned ticket_s;
    __shared__ double edge_out[SLOTS][kEdgeOut];
    __shared__ double hand[kHandDoubles];
    if (blockIdx.x & 1)
        reverse_dp_body<KCH, SLOTS, NPROD>(p, sh, ticket_s, edge_out, hand);
    else
        forward_dp_body<KCH, SLOTS, NPROD>(p, value, sh, ticket_s, edge_out, hand);
}

}  // namespace sdtw
