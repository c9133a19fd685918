// HIP kernels of the Soft-DTW hot path for gfx950.  Included once by sdtw_api.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "device_core.h"
#include "layout.h"

namespace sdtw {

constexpr int kStatusState = 4;    // SDTW_ERR_STATE
constexpr int kStatusTimeout = 6;  // SDTW_ERR_TIMEOUT

// Boundary rows before a sweep: "not written yet" wherever the band that owns the row will publish a
// value.  With a band constraint a sweep skips the macro-steps outside the window; the columns it
// never publishes (forward: the band's last row, columns 32*lo-63 .. 32*hi-32; reverse: its first
// row, columns 32*lo .. 32*hi+31) lie outside the window and hold kBig from the start.
// (blk of nblk: this workgroup's number among those of the launch that share the filling)
__device__ __forceinline__ void fill_boundary_rows(const Params &p, unsigned long long *rows, bool reverse, size_t blk,
                                                   size_t nblk)
{
    const size_t n = (size_t)p.B * p.nbands * p.M;
    const size_t stride = nblk * blockDim.x;
    if (p.window >= kNoWindow && p.x_len == nullptr && p.y_len == nullptr) {
        for (size_t i = blk * blockDim.x + threadIdx.x; i < n; i += stride) rows[i] = kSentinel;
        return;
    }
    const unsigned long long big = (unsigned long long)__double_as_longlong(kBig);
    for (size_t i = blk * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int j = (int)(i % (size_t)p.M);
        const int k = (int)((i / (size_t)p.M) % (size_t)p.nbands);
        const int b = (int)(i / ((size_t)p.M * (size_t)p.nbands));
        const SweepRange r = sweep_range(p, k * kBandRows, k * kBandRows, pair_len_lane(p.x_len, b, p.N),
                                         pair_len_lane(p.y_len, b, p.M));
        const int first = reverse ? kBlk * r.lo : kBlk * r.lo - (kBandRows - 1);
        const int last = reverse ? kBlk * r.hi + kBlk - 1 : kBlk * r.hi - kBlk;
        rows[i] = (r.hi >= r.lo && j >= first && j <= last) ? kSentinel : big;
    }
}

// Start of a forward call, one launch: stamps the header, resets the band tickets, marks every
// boundary value "not written yet", and computes the squared row norms ||x_i||^2, ||y_j||^2
// (Sec. 4.3: the norms are computed once; one wavefront per row, lanes stride over the features).
// The header of a workspace at the start of a forward call (one thread).
__device__ __forceinline__ void stamp_header(const Params &p)
{
    Header *h = p.hdr;
    h->magic = kMagic;
    h->B = p.B; h->N = p.N; h->M = p.M; h->D = p.D; h->mode = p.mode;
    h->gamma_bits = __float_as_uint(p.gamma);
    h->forward_done = 1;
    h->two_sweep = p.two_sweep;
    h->window = p.window;
    h->pieces = p.pieces;
    h->x_len_ptr = reinterpret_cast<uint64_t>(p.x_len);
    h->y_len_ptr = reinterpret_cast<uint64_t>(p.y_len);
    h->status = 0;
    h->abort_backward = 0;
    h->fwd_ticket = 0;
    h->bwd_ticket = 0;
}

// The power of two a row is scaled by before it is split into float16 pieces (largest element in
// [2^13, 2^14)), and its reciprocal.
__device__ __forceinline__ void split_scale(float mx, float &sc, float &inv)
{
    int ex = 0;
    if (mx > 0.f) (void)frexpf(mx, &ex);
    ex = max(-100, min(ex, 120));
    sc = ldexpf(1.0f, 14 - ex);
    inv = ldexpf(1.0f, ex - 14);
}

__global__ __launch_bounds__(256) void forward_prep_kernel(Params p, int64_t xrows, int64_t yrows)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) stamp_header(p);
    fill_boundary_rows(p, p.brow, false, blockIdx.x, gridDim.x);
    if (p.two_sweep) fill_boundary_rows(p, p.brow_b, true, blockIdx.x, gridDim.x);  // the reverse sweep runs in the same call
    const int lane = threadIdx.x & 63;
    const int64_t rows = xrows + yrows;
    const int64_t stride = (int64_t)gridDim.x * 4;
    if (p.Dp > 0 && p.vec_d4) {
        // Rows of up to 128 features, 16-byte loads: a lane takes 4 consecutive features, Dp/4 lanes
        // take a row, a wavefront takes 64/(Dp/4) rows at a time with the next ones in flight.
        // The pieces leave as 8-byte stores.
        const int lpr = p.Dp >> 2, rpw = 64 / lpr;
        const int sub = lane / lpr, k0 = 4 * (lane % lpr);
        auto load_v = [&](int64_t grp) {
            const int64_t row = grp * rpw + sub;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < rows && k0 < p.D)
                v = *reinterpret_cast<const float4 *>((row < xrows ? p.x + row * p.D : p.y + (row - xrows) * p.D) + k0);
            return v;
        };
        const int64_t ngrp = (rows + rpw - 1) / rpw;
        int64_t grp = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        float4 cur = make_float4(0.f, 0.f, 0.f, 0.f);
        if (grp < ngrp) cur = load_v(grp);
        for (; grp < ngrp; grp += stride) {
            float4 nxt = make_float4(0.f, 0.f, 0.f, 0.f);
            if (grp + stride < ngrp) nxt = load_v(grp + stride);
            const int64_t row = grp * rpw + sub;
            const bool isx = row < xrows;
            const int64_t lr = isx ? row : row - xrows;
            float acc = fmaf(cur.x, cur.x, fmaf(cur.y, cur.y, fmaf(cur.z, cur.z, cur.w * cur.w)));
            float mx = fmaxf(fmaxf(fabsf(cur.x), fabsf(cur.y)), fmaxf(fabsf(cur.z), fabsf(cur.w)));
            for (int o = lpr >> 1; o > 0; o >>= 1) {
                acc += __shfl_xor(acc, o);
                mx = fmaxf(mx, __shfl_xor(mx, o));
            }
            int ex = 0;
            if (mx > 0.f) (void)frexpf(mx, &ex);
            ex = max(-100, min(ex, 120));
            const float sc = ldexpf(1.0f, 14 - ex);  // see the comment on the split below
            if (row < rows) {
                if (k0 == 0) {
                    (isx ? p.xn : p.yn)[lr] = acc;
                    (isx ? p.xis : p.yis)[lr] = ldexpf(1.0f, ex - 14);
                }
                typedef _Float16 half4 __attribute__((ext_vector_type(4)));
                half4 h1, h2;
                const float vs[4] = {cur.x * sc, cur.y * sc, cur.z * sc, cur.w * sc};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    h1[c] = (_Float16)vs[c];
                    h2[c] = (_Float16)(vs[c] - (float)h1[c]);
                }
                uint16_t *h = (isx ? p.xh : p.yh) + lr * (2 * p.Dp) + 32 * (k0 >> 4) + (k0 & 15);
                *reinterpret_cast<half4 *>(h) = h1;
                *reinterpret_cast<half4 *>(h + 16) = h2;
            }
            cur = nxt;
        }
        return;
    }
    // One wavefront per row, lanes stride over the features.  Up to 256 features stay in registers
    // and the next row is loaded while the current one is reduced and converted.
    constexpr int kRegs = 4;
    const bool in_regs = p.D <= 64 * kRegs;
    auto row_ptr = [&](int64_t row) { return row < xrows ? p.x + row * p.D : p.y + (row - xrows) * p.D; };
    auto load_row = [&](float (&v)[kRegs], int64_t row) {
        const float *r = row_ptr(row);
#pragma unroll
        for (int c = 0; c < kRegs; ++c) {
            const int k = lane + 64 * c;
            v[c] = (k < p.D) ? r[k] : 0.f;
        }
    };
    float cur[kRegs] = {0.f, 0.f, 0.f, 0.f}, nxt[kRegs] = {0.f, 0.f, 0.f, 0.f};
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (in_regs && row < rows) load_row(cur, row);
    for (; row < rows; row += stride) {
        if (in_regs && row + stride < rows) load_row(nxt, row + stride);
        const bool isx = row < xrows;
        const int64_t lr = isx ? row : row - xrows;
        const float *r = row_ptr(row);
        float acc = 0.f, mx = 0.f;
        if (in_regs) {
#pragma unroll
            for (int c = 0; c < kRegs; ++c) {
                acc = fmaf(cur[c], cur[c], acc);
                mx = fmaxf(mx, fabsf(cur[c]));
            }
        } else {
            for (int k = lane; k < p.D; k += 64) {
                acc = fmaf(r[k], r[k], acc);
                mx = fmaxf(mx, fabsf(r[k]));
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            acc += __shfl_xor(acc, o);
            mx = fmaxf(mx, __shfl_xor(mx, o));
        }
        if (lane == 0) (isx ? p.xn : p.yn)[lr] = acc;
        if (p.Dp > 0) {
            // Split-half copy for the fp16 matrix cores: with a power-of-two scale s that brings the
            // row's largest magnitude into [2^13, 2^14), v*s = h1 + h2 + e with h1, h2 float16 and
            // |e| <= 2^-22 |v*s| (two 11-bit significands).  The products h1*k1 + h1*k2 + h2*k1 then
            // reproduce <x_i, y_j> to about float32 accuracy (the dropped h2*k2 term is ~2^-22 relative).
            // (Dp <= 128, so the row is in registers here.)
            int ex = 0;
            if (mx > 0.f) (void)frexpf(mx, &ex);
            ex = max(-100, min(ex, 120));
            const float sc = ldexpf(1.0f, 14 - ex);
            if (lane == 0) (isx ? p.xis : p.yis)[lr] = ldexpf(1.0f, ex - 14);
            // stored [row][group of 16 features][piece][16]
            uint16_t *h = (isx ? p.xh : p.yh) + lr * (2 * p.Dp);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int k = lane + 64 * c;
                if (k < p.Dp) {
                    const float vs = cur[c] * sc;  // zero beyond D
                    const _Float16 h1 = (_Float16)vs;
                    const _Float16 h2 = (_Float16)(vs - (float)h1);
                    const int o = 32 * (k >> 4) + (k & 15);
                    h[o] = __builtin_bit_cast(uint16_t, h1);
                    h[o + 16] = __builtin_bit_cast(uint16_t, h2);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < kRegs; ++c) cur[c] = nxt[c];
    }
}

// Does the workspace hold the forward of this descriptor?  Every field is read before any is
// compared, and the comparisons are combined without branches: the header costs one memory round
// trip (short-circuit comparisons would take one per field, a microsecond each, at the start of
// kernels that run for ten).
__device__ __forceinline__ bool workspace_matches(const Params &p)
{
    const Header *h = p.hdr;
    const uint32_t magic = h->magic, gamma_bits = h->gamma_bits;
    const int32_t B = h->B, N = h->N, M = h->M, D = h->D, mode = h->mode, done = h->forward_done;
    const int32_t two_sweep = h->two_sweep, window = h->window, pieces = h->pieces;
    const uint64_t xl = h->x_len_ptr, yl = h->y_len_ptr;
    const uint32_t diff = (magic ^ kMagic) | (uint32_t)(done ^ 1) | (uint32_t)(B ^ p.B) | (uint32_t)(N ^ p.N) |
                          (uint32_t)(M ^ p.M) | (uint32_t)(D ^ p.D) | (uint32_t)(mode ^ p.mode) |
                          (uint32_t)(two_sweep ^ p.two_sweep) | (uint32_t)(window ^ p.window) | (uint32_t)(pieces ^ p.pieces) |
                          (gamma_bits ^ __float_as_uint(p.gamma));
    const uint64_t diff_ptr = (xl ^ reinterpret_cast<uint64_t>(p.x_len)) | (yl ^ reinterpret_cast<uint64_t>(p.y_len));
    return (diff == 0) & (diff_ptr == 0);
}

// A backward call's outputs are NaN when the workspace does not match or a sweep gave up waiting.
__device__ __forceinline__ bool backward_refused(const Params &p)
{
    const int32_t aborted = p.hdr->abort_backward, status = p.hdr->status;
    const bool ok = workspace_matches(p);
    return ((aborted | status) != 0) | !ok;
}

// Start of a backward call that runs the reverse sweep itself, one launch: checks that the
// workspace holds the forward of this descriptor, resets the ticket and marks every boundary value
// "not written yet".
__global__ __launch_bounds__(256) void backward_prep_kernel(Params p)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        Header *h = p.hdr;
        const bool ok = workspace_matches(p);
        h->bwd_ticket = 0;
        h->pool_count = 0;
        h->pool_overflow = 0;
        if (ok) {
            h->abort_backward = 0;
        } else {
            h->magic = kMagic;  // make the status word meaningful even on an untouched buffer
            h->forward_done = 0;
            h->abort_backward = 1;
            h->status = kStatusState;
        }
    }
    fill_boundary_rows(p, p.brow_b, true, blockIdx.x, gridDim.x);
    // compact E: every block starts as "all zero"
    if (p.idx != nullptr) {
        const size_t n = (size_t)p.B * p.nrb * p.ncb;
        const size_t stride = (size_t)gridDim.x * blockDim.x;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p.idx[i] = -1;
    }
    // with a band constraint the sweep never visits the blocks of E outside the window: their
    // "any non-zero" flags are cleared here
    if (p.window < kNoWindow || p.x_len != nullptr || p.y_len != nullptr) {
        const size_t n = (size_t)p.B * p.nrb * p.ncb;
        const size_t stride = (size_t)gridDim.x * blockDim.x;
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p.nz[i] = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// Unfused cost tensor d[B,N,M] (Sec. 4.3 "unfused": computed once and stored).
// One workgroup = 4 wavefronts = one 64x64 tile; each wavefront one 32x32 MFMA block.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cost_tensor_kernel(Params p)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int b = blockIdx.z;
    const int i0 = blockIdx.y * 64 + (w >> 1) * 32;
    const int j0 = blockIdx.x * 64 + (w & 1) * 32;
    if (i0 >= p.N || j0 >= p.M) return;
    if (j0 - (i0 + 31) > p.window || i0 - (j0 + 31) > p.window) return;  // no cell of the block is inside the window
    float out[16];
    cost_block(p, p.x + b * p.x_stride, p.y + b * p.y_stride, p.xn + b * p.xn_stride,
               p.yn + b * p.yn_stride, i0, j0, lane, out);
    float *dst = p.cost + (size_t)b * p.N * p.M;
    const int col = j0 + (lane & 31);
    if (col < p.M) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = i0 + acc_row(i, lane);
            if (row < p.N) dst[(size_t)row * p.M + col] = out[i];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Input gradients (Sec. 4.3):  dx_i = 2 g (x_i sum_j E_ij - sum_j E_ij y_j),  dy_j alike.
// One launch covers both: blockIdx.z = 2*b + side.  A workgroup (4 wavefronts) owns a 64 x 64
// output tile (64 sequence positions x 64 features) and walks the other sequence in chunks of 32,
// multiplying the E chunk with the feature chunk on the fp32 matrix cores.  Chunks whose E blocks
// are flagged all-zero are skipped; that changes nothing in the result because a zero E entry
// contributes exactly zero.
//   side 0 (dx): out rows = i, reduction over j;  A[k][m] = E[i0+m][j0+k],  Bv[k][n] = y[j0+k][n0+n]
//   side 1 (dy): out rows = j, reduction over i;  A[k][m] = E[i0+k][j0+m],  Bv[k][n] = x[i0+k][n0+n]
// ---------------------------------------------------------------------------------------------
constexpr int kGradStride = 68;  // floats per LDS row of the k-major 32 x 64 operand tiles

__global__ __launch_bounds__(256) void input_grad_kernel(Params p, const float *__restrict__ grad_value,
                                                        float *__restrict__ dx, float *__restrict__ dy)
{
    __shared__ __attribute__((aligned(16))) float At[kBlk * kGradStride];
    __shared__ __attribute__((aligned(16))) float Bt[kBlk * kGradStride];
    __shared__ float msum_part[4][64];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int b = blockIdx.z >> 1, side = blockIdx.z & 1;
    float *out = side == 0 ? dx : dy;
    if (out == nullptr) return;
    const int P = side == 0 ? p.N : p.M;  // output positions
    const int Q = side == 0 ? p.M : p.N;  // reduced positions
    const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    if (m0 >= P) return;
    // the pair's own lengths (ragged batches): E is zero beyond them, and neither the reduction nor the
    // epilogue reads the sequences' padding
    const int Pl = pair_len(side == 0 ? p.x_len : p.y_len, b, P), Ql = pair_len(side == 0 ? p.y_len : p.x_len, b, Q);
    const float *own = side == 0 ? p.x + b * p.x_stride : p.y + b * p.y_stride;   // sequence of the output side
    const float *oth = side == 0 ? p.y + b * p.y_stride : p.x + b * p.x_stride;   // sequence reduced over
    out += (size_t)b * P * p.D;
    const int wr = w >> 1, wc = w & 1;

    if (backward_refused(p)) {
        const float qnan = __builtin_nanf("");
        for (int e = tid; e < 64 * 64; e += 256) {
            const int m = m0 + (e >> 6), n = n0 + (e & 63);
            if (m < P && n < p.D) out[(size_t)m * p.D + n] = qnan;
        }
        return;
    }

    const float *Eb = p.E + (size_t)b * p.N * p.M;
    const unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float msum = 0.f;  // thread (w, lane): partial sum of E over the reduced index for output row m0+lane

    // which of the two 32x32 E blocks of the chunk at q0 have a non-zero?  (bit 0: the first 32 output
    // positions, bit 1: the other 32.)  A block whose flag is clear is never read: it is all zero by
    // definition, and nobody may have written it.
    auto chunk_flags = [&](int q0) {
        const int qb = q0 / kBlk, mb = m0 / kBlk;
        int bits;
        if (side == 0) {
            bits = nzb[(size_t)mb * p.ncb + qb] != 0 ? 1 : 0;
            if (mb + 1 < p.nrb && nzb[(size_t)(mb + 1) * p.ncb + qb] != 0) bits |= 2;
        } else {
            bits = nzb[(size_t)qb * p.ncb + mb] != 0 ? 1 : 0;
            if (mb + 1 < p.ncb && nzb[(size_t)qb * p.ncb + mb + 1] != 0) bits |= 2;
        }
        return bits;
    };
    int live_bits = 0;  // flags of the chunk next_live stopped at
    auto next_live = [&](int q0) {
        live_bits = 0;
        while (q0 < Ql && (live_bits = chunk_flags(q0)) == 0) q0 += kBlk;
        return q0;
    };
    auto load4 = [](const float *q, int first, int limit, bool vec) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vec && first + 3 < limit) {
            t = *reinterpret_cast<const float4 *>(q);
        } else {
            if (first + 0 < limit) t.x = q[0];
            if (first + 1 < limit) t.y = q[1];
            if (first + 2 < limit) t.z = q[2];
            if (first + 3 < limit) t.w = q[3];
        }
        return t;
    };
    // A chunk's operands travel global -> registers -> LDS; the loads of the next chunk are issued
    // before the matrix-core work of the current one.  Per thread: two float4 of E, two of the sequence.
    //   side 0: E rows i = m0+m (64), columns j = q0+k (32): element e -> m = e/8, k = 4*(e%8)
    //   side 1: E rows i = q0+k (32), columns j = m0+m (64): element e -> k = e/16, m = 4*(e%16)
    float4 ra[2], rb[2];
    auto fetch = [&](int q0) {
        const int bits = live_bits;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int e = tid + 256 * r;
            ra[r] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (side == 0) {
                const int i = m0 + (e >> 3), k4 = (e & 7) * 4;  // rows m0 .. m0+31 for r = 0, the other 32 for r = 1
                if (i < p.N && ((bits >> r) & 1)) ra[r] = load4(Eb + (size_t)i * p.M + q0 + k4, q0 + k4, p.M, p.vec_m != 0);
            } else {
                const int i = q0 + (e >> 4), m4 = (e & 15) * 4;  // columns m0 .. m0+31 for m4 < 32
                if (i < p.N && ((bits >> (m4 >> 5)) & 1)) ra[r] = load4(Eb + (size_t)i * p.M + m0 + m4, m0 + m4, p.M, p.vec_m != 0);
            }
            const int q = q0 + (e >> 4), n4 = (e & 15) * 4;
            rb[r] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (q < Ql) rb[r] = load4(oth + (size_t)q * p.D + n0 + n4, n0 + n4, p.D, p.vec_xy != 0);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int e = tid + 256 * r;
            if (side == 0) {  // k-major: At[k][m]
                const int m = e >> 3, k4 = (e & 7) * 4;
                At[(k4 + 0) * kGradStride + m] = ra[r].x;
                At[(k4 + 1) * kGradStride + m] = ra[r].y;
                At[(k4 + 2) * kGradStride + m] = ra[r].z;
                At[(k4 + 3) * kGradStride + m] = ra[r].w;
            } else {
                *reinterpret_cast<float4 *>(At + (e >> 4) * kGradStride + (e & 15) * 4) = ra[r];
            }
            *reinterpret_cast<float4 *>(Bt + (e >> 4) * kGradStride + (e & 15) * 4) = rb[r];
        }
    };

    int q0 = next_live(0);
    if (q0 < Ql) fetch(q0);
    while (q0 < Ql) {
        __syncthreads();  // previous chunk's reads are done
        stash();
        __syncthreads();
        q0 = next_live(q0 + kBlk);
        if (q0 < Ql) fetch(q0);

        // marginal sums: wavefront w adds rows k = 8w .. 8w+7 of the A tile for output row `lane`
#pragma unroll
        for (int k = 0; k < 8; ++k) msum += At[(8 * w + k) * kGradStride + lane];

        const int am = wr * 32 + (lane & 31), bn = wc * 32 + (lane & 31), kh = lane >> 5;
#pragma unroll
        for (int k2 = 0; k2 < kBlk; k2 += 2) {
            const float a = At[(k2 + kh) * kGradStride + am];
            const float bv = Bt[(k2 + kh) * kGradStride + bn];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc, 0, 0, 0);
        }
    }

    msum_part[w][lane] = msum;
    __syncthreads();
    const float scale = 2.0f * (grad_value ? grad_value[b] : 1.0f);
    const int n = n0 + wc * 32 + (lane & 31);
    if (n < p.D) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ml = wr * 32 + acc_row(i, lane);
            const int m = m0 + ml;
            if (m < P) {
                const float tot = (msum_part[0][ml] + msum_part[1][ml]) + (msum_part[2][ml] + msum_part[3][ml]);
                const float ov = m < Pl ? own[(size_t)m * p.D + n] : 0.f;
                out[(size_t)m * p.D + n] = scale * (ov * tot - acc[i]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Input gradients for D <= 128 on the fp16 matrix cores (same formulas, Sec. 4.3).
// Both operands of  sum_q E[m,q] * oth[q,n]  are split into two float16 pieces: E * 2^10 (entries
// in [0,1]) and oth * s with one power-of-two scale s per chunk of 32 reduced positions that brings
// the chunk's largest magnitude into [2^13, 2^14) (from the per-row scales the forward call
// stored); a chunk's products are accumulated from zero and added to the total with 1/(2^10 s).  With
// a = a1 + a2, b = b1 + b2 the product is a1*b1 + a1*b2 + a2*b1 (the dropped a2*b2 is ~2^-22
// relative), accumulated in float32 by v_mfma_f32_32x32x16_f16; the marginal sums of E are added up
// in float32 from the unsplit values.  Tiles, zero-block skipping and the epilogue are those of
// input_grad_kernel; the pieces sit in LDS as [row][32 reduced positions] with 80-byte rows, so that
// a lane's 8 consecutive reduced positions are one 16-byte read.
// ---------------------------------------------------------------------------------------------
constexpr int kLiveCap = 1024;     // chunks listed at a time (with the pool positions: 12 KB of LDS)
constexpr int kGradHalfRow = 40;  // float16 per LDS row: 32 used, padded to 80 bytes against bank conflicts

__device__ __forceinline__ void split8(const float (&v)[8], float scale, half8 &h1, half8 &h2)
{
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float vs = v[c] * scale;
        const _Float16 a = (_Float16)vs;
        h1[c] = a;
        h2[c] = (_Float16)(vs - (float)a);
    }
}

__global__ __launch_bounds__(256) void input_grad_half_kernel(Params p, const float *__restrict__ grad_value,
                                                             float *__restrict__ dx, float *__restrict__ dy)
{
    __shared__ __attribute__((aligned(16))) _Float16 Ah[2][2][64 * kGradHalfRow];  // [buffer][piece][m][k]
    __shared__ __attribute__((aligned(16))) _Float16 Bh[2][2][64 * kGradHalfRow];  // [buffer][piece][n][k]
    __shared__ float msum_part[4][64];
    __shared__ int live_list[kLiveCap];          // first reduced position of every chunk that has a non-zero
    __shared__ int live_slot[2][kLiveCap];       // compact E: where the chunk's two blocks lie in the pool (-1: all zero)
    __shared__ unsigned long long wave_mask[2][4];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int b = blockIdx.z >> 1, side = blockIdx.z & 1;
    float *out = side == 0 ? dx : dy;
    if (out == nullptr) return;
    const int P = side == 0 ? p.N : p.M;  // output positions
    const int Q = side == 0 ? p.M : p.N;  // reduced positions
    const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    if (m0 >= P) return;
    // the pair's own lengths (ragged batches): E is zero beyond them, and neither the reduction nor the
    // epilogue reads the sequences' padding
    const int Pl = pair_len(side == 0 ? p.x_len : p.y_len, b, P), Ql = pair_len(side == 0 ? p.y_len : p.x_len, b, Q);
    const float *own = side == 0 ? p.x + b * p.x_stride : p.y + b * p.y_stride;   // sequence of the output side
    const float *oth = side == 0 ? p.y + b * p.y_stride : p.x + b * p.x_stride;   // sequence reduced over
    // its rows' 1/scale (positive powers of two: their bit patterns order like the values)
    const unsigned *oth_is = reinterpret_cast<const unsigned *>(side == 0 ? p.yis + b * p.yn_stride : p.xis + b * p.xn_stride);
    out += (size_t)b * P * p.D;
    const int wr = w >> 1, wc = w & 1;

    // (the header is asked for now and looked at below, once the first flags and the output side's
    // own values have been asked for as well: one wait for all three)
    const bool refused = backward_refused(p);
    // compact E: the blocks lie in the pool (32 x 32 row-major each, found through the index); if the pool
    // ran over, the gradients come from the second sweep instead and this kernel has nothing to do
    const bool pooled = p.idx != nullptr;
    const int32_t *idxb = pooled ? p.idx + (size_t)b * p.nrb * p.ncb : nullptr;
    const int32_t overflow = pooled ? p.hdr->pool_overflow : 0;  // (looked at below, with the rest of the header)

    const float sA = 1024.0f;
    // the largest 1/scale among the chunk's 32 rows: one row per lane (mod 32; both halves of the
    // wavefront hold the same 32), then the maximum over the wavefront by lane shifts
    auto chunk_ismax = [&](int q0) { return wave_max_f32(__uint_as_float(oth_is[min(q0 + (lane & 31), Ql - 1)])); };

    const float *Eb = p.E + (size_t)b * p.N * p.M;
    const unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;
    floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const floatx16 zero = acc;
    float msum = 0.f;  // partial sum of E over the reduced index for one output row (which: see stash)

    // which of the two 32x32 E blocks of the chunk at q0 have a non-zero?  (bit 0: the first 32 output
    // positions, bit 1: the other 32.)  A block whose flag is clear is never read: it is all zero by
    // definition, and nobody may have written it.
    auto chunk_flags = [&](int q0) {
        const int qb = q0 / kBlk, mb = m0 / kBlk;
        unsigned bits;
        if (side == 0) {
            bits = nzb[(size_t)mb * p.ncb + qb] != 0 ? 1u : 0u;
            if (mb + 1 < p.nrb && nzb[(size_t)(mb + 1) * p.ncb + qb] != 0) bits |= 2u;
        } else {
            bits = nzb[(size_t)qb * p.ncb + mb] != 0 ? 1u : 0u;
            if (mb + 1 < p.ncb && nzb[(size_t)qb * p.ncb + mb + 1] != 0) bits |= 2u;
        }
        return bits;
    };
    // compact E: the same from the block index (a block is live where it has a pool position), which is
    // what the list needs anyway: one memory round trip instead of flags first and positions after
    auto chunk_slots = [&](int q0, int &s0, int &s1) {
        const int qb = q0 / kBlk, mb = m0 / kBlk;
        s1 = -1;
        if (side == 0) {
            s0 = idxb[(size_t)mb * p.ncb + qb];
            if (mb + 1 < p.nrb) s1 = idxb[(size_t)(mb + 1) * p.ncb + qb];
        } else {
            s0 = idxb[(size_t)qb * p.ncb + mb];
            if (mb + 1 < p.ncb) s1 = idxb[(size_t)qb * p.ncb + mb + 1];
        }
        return (s0 >= 0 ? 1u : 0u) | (s1 >= 0 ? 2u : 0u);
    };

    // Per thread and chunk: 8 values of E and 8 of the reduced sequence, each run along the reduced
    // index k (the fast index of the LDS rows).
    //   side 0, E rows i = m0+m, columns q0+k:  m = tid/4, k = 8*(tid%4) .. +7  (32 contiguous bytes)
    //   side 1, E rows q0+k, columns j = m0+m:  m = tid%64, k = 8*(tid/64) .. +7  (8 rows, lanes along j)
    //   sequence rows q0+k, features n0+n:      n = tid%64, k = 8*(tid/64) .. +7
    const int am = side == 0 ? (tid >> 2) : lane, ak = side == 0 ? (tid & 3) * 8 : w * 8;
    const int bn = lane, bk = w * 8;
    // (a list entry is the chunk's first reduced position with the two block flags in bits 30 and 31)
    auto fetch = [&](int pos, float (&ea)[8], float (&bv)[8], float &ismax) {
        const int entry = live_list[pos];
        const int q0 = entry & 0x3FFFFFFF;
        const bool blk_live = (((unsigned)entry >> (30 + (am >> 5))) & 1u) != 0;  // the block this thread's output position is in
        ismax = chunk_ismax(q0);
        // this thread's block of E: rows of M floats in the dense tensor, of 32 in a pool block
        const float *blk = nullptr;
        if (pooled && blk_live) blk = p.pool + (size_t)live_slot[am >> 5][pos] * (kBlk * kBlk);
        const size_t ld = pooled ? (size_t)kBlk : (size_t)p.M;
        if (side == 0) {
            const int i = m0 + am;
#pragma unroll
            for (int c = 0; c < 8; ++c) ea[c] = 0.f;
            if (i < p.N && blk_live) {
                const float *q = pooled ? blk + (size_t)(i & (kBlk - 1)) * kBlk + ak : Eb + (size_t)i * p.M + q0 + ak;
                if ((pooled || p.vec_m) && q0 + ak + 7 < p.M) {
                    const float4 t0 = *reinterpret_cast<const float4 *>(q), t1 = *reinterpret_cast<const float4 *>(q + 4);
                    ea[0] = t0.x; ea[1] = t0.y; ea[2] = t0.z; ea[3] = t0.w;
                    ea[4] = t1.x; ea[5] = t1.y; ea[6] = t1.z; ea[7] = t1.w;
                } else {
#pragma unroll
                    for (int c = 0; c < 8; ++c) if (q0 + ak + c < p.M) ea[c] = q[c];
                }
            }
        } else {
            const int j = m0 + am;
            const float *e = pooled ? blk + (size_t)ak * kBlk + (j & (kBlk - 1)) : Eb + (size_t)(q0 + ak) * p.M + j;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int i = q0 + ak + c;
                ea[c] = (i < p.N && j < p.M && blk_live) ? *e : 0.f;
                e += ld;
            }
        }
        const int n = n0 + bn;
        const float *o = oth + (size_t)(q0 + bk) * p.D + n;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int q = q0 + bk + c;
            bv[c] = (q < Ql && n < p.D) ? *o : 0.f;
            o += p.D;
        }
    };
    auto stash = [&](int buf, const float (&ea)[8], const float (&bv)[8], float ismax) {
        half8 h1, h2;
        const float sB = 1.0f / ismax;  // exact: a power of two
        split8(ea, sA, h1, h2);
        *reinterpret_cast<half8 *>(&Ah[buf][0][am * kGradHalfRow + ak]) = h1;
        *reinterpret_cast<half8 *>(&Ah[buf][1][am * kGradHalfRow + ak]) = h2;
        split8(bv, sB, h1, h2);
        *reinterpret_cast<half8 *>(&Bh[buf][0][bn * kGradHalfRow + bk]) = h1;
        *reinterpret_cast<half8 *>(&Bh[buf][1][bn * kGradHalfRow + bk]) = h2;
        // marginal sums from the unsplit values: this thread's 8 entries of output row `am`
        msum += ((ea[0] + ea[1]) + (ea[2] + ea[3])) + ((ea[4] + ea[5]) + (ea[6] + ea[7]));
    };
    // the matrix-core work of one chunk, added to the total with the chunk's scale undone
    auto contract = [&](int buf, float ismax) {
        const int ar = (wr * 32 + (lane & 31)) * kGradHalfRow, br = (wc * 32 + (lane & 31)) * kGradHalfRow;
        const int kh = (lane >> 5) * 8;
        floatx16 part = zero;
#pragma unroll
        for (int ks = 0; ks < kBlk; ks += 16) {
            const half8 a1 = *reinterpret_cast<const half8 *>(&Ah[buf][0][ar + ks + kh]);
            const half8 a2 = *reinterpret_cast<const half8 *>(&Ah[buf][1][ar + ks + kh]);
            const half8 b1 = *reinterpret_cast<const half8 *>(&Bh[buf][0][br + ks + kh]);
            const half8 b2 = *reinterpret_cast<const half8 *>(&Bh[buf][1][br + ks + kh]);
            part = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b1, part, 0, 0, 0);
            part = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b2, part, 0, 0, 0);
            part = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, b1, part, 0, 0, 0);
        }
        const float unscale = ismax * (1.0f / 1024.0f);
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = fmaf(part[i], unscale, acc[i]);
    };

    // The chunks are examined kLiveCap at a time: first, 256 per round, every thread reads the flags
    // of one chunk and the live ones are listed in order (ballot + prefix counts, so the order and
    // with it the rounding never changes); then the listed chunks are contracted with two of them in
    // flight: while chunk c is contracted, the values of chunk c+1 are arriving and those of chunk
    // c+2 are requested.
    const int nchunk = (Ql + kBlk - 1) / kBlk;
    // the output side's own values for the epilogue, requested now so that they are there by then
    float own_v[16];
    {
        // (addresses by adding the row length up: a multiplication per element would cost a lone
        // wavefront more than the loads themselves)
        const int n = n0 + wc * 32 + (lane & 31);
        const int mb = m0 + wr * 32 + 4 * (lane >> 5);
        const float *og = own + (size_t)mb * p.D + n;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const float *o = og;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int m = mb + 8 * g4 + k;  // == m0 + wr*32 + acc_row(4*g4 + k, lane)
                own_v[4 * g4 + k] = (m < Pl && n < p.D) ? *o : 0.f;
                o += p.D;
            }
            og += 8 * (size_t)p.D;
        }
    }
    int first_s0 = -1, first_s1 = -1;
    unsigned first_bits = 0u;
    if (tid < min(nchunk, kLiveCap)) first_bits = pooled ? chunk_slots(tid * kBlk, first_s0, first_s1) : chunk_flags(tid * kBlk);
    if (refused) {
        const float qnan = __builtin_nanf("");
        for (int e = tid; e < 64 * 64; e += 256) {
            const int m = m0 + (e >> 6), n = n0 + (e & 63);
            if (m < P && n < p.D) out[(size_t)m * p.D + n] = qnan;
        }
        return;
    }
    if (overflow != 0) return;
    float ea0[8], bv0[8], ea1[8], bv1[8], is0 = 1.f, is1 = 1.f;
    for (int base = 0; base < nchunk; base += kLiveCap) {
        const int lim = min(nchunk, base + kLiveCap);
        int nlive = 0;
        for (int g = base, round = 0; g < lim; g += 256, ++round) {
            const int c = g + tid;
            int s0 = first_s0, s1 = first_s1;
            unsigned bits = first_bits;
            if (g != 0) {
                s0 = s1 = -1;
                bits = c < lim ? (pooled ? chunk_slots(c * kBlk, s0, s1) : chunk_flags(c * kBlk)) : 0u;
            }
            const bool lv = bits != 0;
            const unsigned long long m = __ballot(lv);
            if (lane == 0) wave_mask[round & 1][w] = m;
            __syncthreads();
            int off = nlive, total = 0;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                const int cnt = __popcll(wave_mask[round & 1][ww]);
                if (ww < w) off += cnt;
                total += cnt;
            }
            if (lv) {
                const int pos = off + __popcll(m & ((1ull << lane) - 1ull));
                live_list[pos] = (int)((unsigned)(c * kBlk) | (bits << 30));
                if (pooled) {
                    live_slot[0][pos] = s0;
                    live_slot[1][pos] = s1;
                }
            }
            nlive += total;
        }
        __syncthreads();

        int i = 0;
        if (nlive > 0) fetch(0, ea0, bv0, is0);
        if (nlive > 1) fetch(1, ea1, bv1, is1);
        // (two LDS buffers, one barrier per chunk: a buffer is written again two chunks later, after
        // the barrier of the chunk in between, by when every wavefront is done reading it)
        while (i < nlive) {
            stash(0, ea0, bv0, is0);
            const float isc0 = is0;
            __syncthreads();
            if (i + 2 < nlive) fetch(i + 2, ea0, bv0, is0);
            contract(0, isc0);
            if (++i >= nlive) break;

            stash(1, ea1, bv1, is1);
            const float isc1 = is1;
            __syncthreads();
            if (i + 2 < nlive) fetch(i + 2, ea1, bv1, is1);
            contract(1, isc1);
            ++i;
        }
        __syncthreads();  // the list is rebuilt next
    }

    // side 0: four threads (tid%4) hold parts of row tid/4; side 1: four wavefronts hold parts of row tid%64
    msum_part[side == 0 ? (tid & 3) : w][am] = msum;
    __syncthreads();
    const float scale = 2.0f * (grad_value ? grad_value[b] : 1.0f);
    const int n = n0 + wc * 32 + (lane & 31);
    if (n < p.D) {
        const int mlb = wr * 32 + 4 * (lane >> 5);
        float *og = out + (size_t)(m0 + mlb) * p.D + n;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            float *o = og;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = 4 * g4 + k, ml = mlb + 8 * g4 + k;  // ml == wr*32 + acc_row(i, lane)
                if (m0 + ml < P) {
                    const float tot = (msum_part[0][ml] + msum_part[1][ml]) + (msum_part[2][ml] + msum_part[3][ml]);
                    *o = scale * (own_v[i] * tot - acc[i]);
                }
                o += p.D;
            }
            og += 8 * (size_t)p.D;
        }
    }
}

// Compact E whose pool ran over: start of the second reverse sweep, the one that contracts E into the
// gradients itself.  Does nothing unless the overflow flag is up; otherwise resets the band tickets,
// marks every boundary value of the reverse sweep "not written yet" again and clears the sums that
// sweep adds to (they lie where the pool was: nobody reads the pool any more).
__global__ __launch_bounds__(256) void second_sweep_prep_kernel(Params p)
{
    static_assert(sizeof(Params) <= 1024, "room for the parameter block in the workspace");
    if (p.hdr->pool_overflow == 0 || p.hdr->abort_backward != 0) return;
    if (threadIdx.x == 0 && blockIdx.x == 0) *const_cast<Params *>(p.self) = p;
    if (threadIdx.x == 0 && blockIdx.x == 0) p.hdr->bwd_ticket = 0;
    fill_boundary_rows(p, p.brow_b, true, blockIdx.x, gridDim.x);
    const size_t stride = (size_t)gridDim.x * blockDim.x, first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    auto clear = [&](float *dst, size_t n) {  // dst is 16-byte aligned (caller's tensors, workspace regions)
        if (dst == nullptr) return;
        for (size_t i = first; i < n / 4; i += stride) reinterpret_cast<float4 *>(dst)[i] = z4;
        for (size_t i = (n / 4) * 4 + first; i < n; i += stride) dst[i] = 0.f;
    };
    clear(p.gdx, (size_t)p.B * p.N * p.D);
    clear(p.rsum, (size_t)p.B * p.N);
    if (p.gdy != nullptr) {  // (integer words: all bits zero, like 0.f)
        clear(p.gdy, (size_t)p.B * p.M * p.D);
        clear(reinterpret_cast<float *>(p.gdy_hi), (size_t)p.B * p.M * p.D);
        clear(reinterpret_cast<float *>(p.csum_lo), (size_t)p.B * p.M);
        clear(reinterpret_cast<float *>(p.csum_hi), (size_t)p.B * p.M);
    }
}

// Exponent bound of every pair's x for the fixed-point sums of the y side (Params::gdy_hi):
// pair_exp[b] = e with |x_b[i][k]| < 2^e for all rows of the pair, read off the per-row scales
// 2^(e_row - 14) that the forward call stored with the split copies.  One workgroup per pair.
__global__ __launch_bounds__(256) void pair_exponent_kernel(Params p, int32_t *__restrict__ pair_exp)
{
    __shared__ unsigned part[4];
    if (p.hdr->pool_overflow == 0) return;
    const int b = blockIdx.x;
    const int Nl = pair_len(p.x_len, b, p.N);
    const unsigned *is = reinterpret_cast<const unsigned *>(p.xis + b * p.xn_stride);
    unsigned m = 0u;  // positive powers of two: their bit patterns order like the values
    for (int i = threadIdx.x; i < Nl; i += 256) m = max(m, is[i]);
    const float mw = wave_max_f32(__uint_as_float(m));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = __float_as_uint(mw);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned bits = max(max(part[0], part[1]), max(part[2], part[3]));
        pair_exp[b] = (int32_t)((bits >> 23) & 255u) - 127 + 14;
    }
}

// After the second reverse sweep of a compact layout (the one that contracts E into the gradients
// itself; it only ran if the pool overflowed, and this kernel only acts then): gdx holds sum_j E_ij y_j, rsum
// sum_j E_ij; gdy / gdy_hi and csum_lo / csum_hi hold sum_i E_ij x_i and sum_i E_ij in fixed point
// (see Params).  The formulas of Sec. 4.3 are completed in place,
//   dx_i = 2 g (x_i sum_j E_ij - sum_j E_ij y_j),   dy_j = 2 g (y_j sum_i E_ij - sum_i E_ij x_i),
// with zeros beyond a pair's own lengths (the sequences' padding is not read) and NaN when the
// backward call was refused.  One thread per W consecutive features (W = 4 needs D % 4 == 0 and
// 16-byte aligned tensors).
template <int W>
__global__ __launch_bounds__(256) void gradient_finish_kernel(Params p, const float *__restrict__ grad_value)
{
    const bool bad = backward_refused(p);
    if (p.hdr->pool_overflow == 0 && !bad) return;  // input_grad_half_kernel wrote the gradients from the pool
    const float qnan = __builtin_nanf("");
    const size_t nx = (size_t)p.B * p.N * p.D, ny = (size_t)p.B * p.M * p.D;
    const size_t stride = (size_t)gridDim.x * blockDim.x * W;
    const double lo_unit = (double)(1ll << p.fx_lo_bits);
    for (size_t e = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * W; e < nx + ny; e += stride) {
        const bool isx = e < nx;
        float *g = isx ? p.gdx : p.gdy;
        if (g == nullptr) continue;
        const size_t q = isx ? e : e - nx;           // element of [B, P, D]
        const int P = isx ? p.N : p.M;
        const size_t row = q / (size_t)p.D;          // b * P + position
        const int b = (int)(row / (size_t)P), pos = (int)(row - (size_t)b * P);
        const int len = pair_len_lane(isx ? p.x_len : p.y_len, b, P);
        const float *seq = (isx ? p.x + b * p.x_stride : p.y + b * p.y_stride) + (size_t)pos * p.D + (q - row * p.D);
        const float scale = 2.0f * (grad_value ? grad_value[b] : 1.0f);
        const bool in = pos < len;
        float acc[W], sv[W], marg;
        if (isx) {
            marg = p.rsum[row];
#pragma unroll
            for (int c = 0; c < W; ++c) acc[c] = g[q + c];
        } else {
            marg = (float)ldexp((double)p.csum_hi[row] * lo_unit + (double)p.csum_lo[row], -24);
            const unsigned *lo = reinterpret_cast<const unsigned *>(g);
            const int ex = p.pair_exp[b] - p.fx_prec;
#pragma unroll
            for (int c = 0; c < W; ++c) acc[c] = (float)ldexp((double)p.gdy_hi[q + c] * lo_unit + (double)lo[q + c], ex);
        }
#pragma unroll
        for (int c = 0; c < W; ++c) sv[c] = in ? seq[c] : 0.f;
#pragma unroll
        for (int c = 0; c < W; ++c) {
            const float o = in ? scale * (sv[c] * marg - acc[c]) : 0.f;
            g[q + c] = bad ? qnan : o;
        }
    }
}

// Where the caller supplied the memory for E (large problems, E_out): the sweep wrote the blocks that
// hold a non-zero straight into it; this fills in the rest (zeros; NaN when the call was refused).
__global__ void complete_E_kernel(Params p)
{
    const size_t n = (size_t)p.B * p.N * p.M;
    const bool bad = backward_refused(p);
    const float qnan = __builtin_nanf("");
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; e < n; e += stride) {
        const int j = (int)(e % (size_t)p.M);
        const size_t bi = e / (size_t)p.M;
        const int i = (int)(bi % (size_t)p.N);
        const size_t b = bi / (size_t)p.N;
        const bool live = p.nz[(b * p.nrb + i / kBlk) * p.ncb + j / kBlk] != 0;
        if (bad)
            p.E[e] = qnan;
        else if (!live)
            p.E[e] = 0.f;
    }
}

// Copies E to the caller's buffer (NaN when the backward call was refused).  A 32x32 block whose
// "any non-zero" flag is clear is all zero by definition; with a band constraint the blocks outside
// the window have never been written.
__global__ void export_E_kernel(Params p, float *__restrict__ dst)
{
    const size_t n = (size_t)p.B * p.N * p.M;
    const bool bad = backward_refused(p);
    const float qnan = __builtin_nanf("");
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; e < n; e += stride) {
        const int j = (int)(e % (size_t)p.M);
        const size_t bi = e / (size_t)p.M;
        const int i = (int)(bi % (size_t)p.N);
        const size_t b = bi / (size_t)p.N;
        const bool live = p.nz[(b * p.nrb + i / kBlk) * p.ncb + j / kBlk] != 0;
        dst[e] = bad ? qnan : (live ? p.E[e] : 0.f);
    }
}

// Un-skews the step-major DP table into row-major R[b][i][j], in the paper's units (test hook).
__global__ void export_R_kernel(Params p, double *__restrict__ dst)
{
    const size_t n = (size_t)p.B * p.N * p.M;
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t band_elems = (size_t)p.nm_tab * kBlk * kBandRows;
    for (; e < n; e += stride) {
        const int j = (int)(e % p.M);
        const size_t bi = e / p.M;
        const int i = (int)(bi % p.N);
        const int b = (int)(bi / p.N);
        const int k = i / kBandRows, t = i % kBandRows;
        const int sg = (j + t) / kBlk - table_base(p, k);  // macro-step within the band's table
        dst[e] = (sg < 0 || sg >= p.nm_tab) ? __builtin_inf()
                                            : p.R[((size_t)b * p.nbands + k) * band_elems +
                                                  ((size_t)sg * kBlk + (j + t) % kBlk) * kBandRows + t] * p.inv_c2d;
    }
}

// ---------------------------------------------------------------------------------------------
// Normalised Soft-DTW (Sec. 6): combination of the cross term and the two self terms.
// ---------------------------------------------------------------------------------------------
// value[b] = xy[b] - (xx[bx] + yy[by]) / 2; a shared sequence has one self term (index 0)
__global__ void normalized_value_kernel(float *__restrict__ value, const float *__restrict__ vxy,
                                        const float *__restrict__ vxx, const float *__restrict__ vyy, int B,
                                        int x_shared, int y_shared)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) value[b] = vxy[b] - 0.5f * (vxx[x_shared ? 0 : b] + vyy[y_shared ? 0 : b]);
}

// g[b][e] -= grad_value[b] * self[b or 0][e]: the self term's gradient with respect to its first
// argument (computed with upstream gradient 1) is the gradient of half the self term.
__global__ void normalized_grad_kernel(float *__restrict__ g, const float *__restrict__ self,
                                       const float *__restrict__ grad_value, int B, int64_t per_pair, int shared)
{
    const int64_t n = (int64_t)B * per_pair;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int64_t b = i / per_pair, e = i - b * per_pair;
        const float gv = grad_value ? grad_value[b] : 1.0f;
        g[i] -= gv * self[(shared ? 0 : b) * per_pair + e];
    }
}

// Normalised Soft-DTW as one batch of 3B pairs (equal lengths, nothing shared): pairs 0..B-1 are
// (x_b, y_b), B..2B-1 are (x_b, x_b), 2B..3B-1 are (y_b, y_b).  This kernel lays the operands out
// that way (per sequence `per` floats, a multiple of 4 or copied one by one).
__global__ void normalized_gather_kernel(const float *__restrict__ x, const float *__restrict__ y, int64_t x_stride,
                                         int64_t y_stride, float *__restrict__ xs, float *__restrict__ ys, int B,
                                         int64_t per, int vec)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (vec) {
        const int64_t per4 = per / 4, n = 3 * (int64_t)B * per4;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
            const int64_t q = i / per4, e = i - q * per4;
            const int kind = (int)(q / B), b = (int)(q - (int64_t)kind * B);
            const float4 xv = reinterpret_cast<const float4 *>(x + b * x_stride)[e];
            const float4 yv = reinterpret_cast<const float4 *>(y + b * y_stride)[e];
            reinterpret_cast<float4 *>(xs)[i] = kind == 2 ? yv : xv;
            reinterpret_cast<float4 *>(ys)[i] = kind == 1 ? xv : yv;
        }
    } else {
        const int64_t n = 3 * (int64_t)B * per;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
            const int64_t q = i / per, e = i - q * per;
            const int kind = (int)(q / B), b = (int)(q - (int64_t)kind * B);
            const float xv = x[b * x_stride + e], yv = y[b * y_stride + e];
            xs[i] = kind == 2 ? yv : xv;
            ys[i] = kind == 1 ? xv : yv;
        }
    }
}

// ... and this one forms the gradients from the batch's (computed with upstream gradient 1):
// dx_b = g_b (d/dx of the cross term - d/d(first argument) of the (x,x) term), dy_b alike with (y,y):
// the self terms are symmetric, so the gradient of half of one is its first-argument gradient.
__global__ void normalized_batched_grad_kernel(float *__restrict__ dx, float *__restrict__ dy,
                                               const float *__restrict__ dxs, const float *__restrict__ dys,
                                               const float *__restrict__ grad_value, int B, int64_t per)
{
    const int64_t n = (int64_t)B * per;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int64_t b = i / per;
        const float gv = grad_value ? grad_value[b] : 1.0f;
        if (dx) dx[i] = gv * (dxs[i] - dxs[n + i]);
        if (dy) dy[i] = gv * (dys[i] - dxs[2 * n + i]);
    }
}

// the cross term's header reports the worst status of the three workspaces
__global__ void merge_status_kernel(Header *xy, const Header *xx, const Header *yy)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int st = xy->status;
        if (xx->magic == kMagic) st = max(st, xx->status);
        if (yy->magic == kMagic) st = max(st, yy->status);
        xy->status = st;
    }
}

// ---------------------------------------------------------------------------------------------
// Reduced-precision inputs (Sec. 6, "Mixed precision"): float16 or bfloat16 sequences are widened to
// float32 copies in the workspace (exact), which the other kernels then read like any float32 input.
// ---------------------------------------------------------------------------------------------
__global__ void widen_half_kernel(const uint16_t *__restrict__ src, float *__restrict__ dst, size_t n, int bf16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint16_t h = src[i];
        dst[i] = bf16 ? __uint_as_float((unsigned)h << 16) : (float)__builtin_bit_cast(_Float16, h);
    }
}

// ---------------------------------------------------------------------------------------------
// Barycenter step (Sec. 4.4): reduce over the K pairs, then Adam.
// ---------------------------------------------------------------------------------------------
struct AdamParams {
    int K;
    int64_t n;  // Lz*D
    float lr, beta1, beta2, eps;
    float corr1, corr2;  // 1-beta1^step, 1-beta2^step
};

// When the pair workspace reports an error (a band gave up waiting, or the workspace did not match),
// the gradients are NaN: loss and dz_out receive them, but z and the optimiser state are left as
// they were, so that the caller can read the status word and retry.
__global__ void barycenter_update_kernel(AdamParams a, const Header *__restrict__ hdr,
                                         const float *__restrict__ dxk /*[K][n]*/,
                                         const float *__restrict__ values /*[K]*/, float *__restrict__ z,
                                         float *__restrict__ m, float *__restrict__ v,
                                         float *__restrict__ loss, float *__restrict__ dz_out)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool failed = (hdr->status | hdr->abort_backward) != 0;
    // sums over k in index order; the loads of 16 terms are asked for together (one memory round trip
    // per 16 sequences instead of one per sequence)
    constexpr int kBatch = 16;
    if (q == 0) {
        float L = 0.f;
        for (int k0 = 0; k0 < a.K; k0 += kBatch) {
            float t[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) t[i] = k0 + i < a.K ? values[k0 + i] : 0.f;
#pragma unroll
            for (int i = 0; i < kBatch; ++i) L += t[i];
        }
        loss[0] = L;
    }
    if (q >= a.n) return;
    float g = 0.f;
    for (int k0 = 0; k0 < a.K; k0 += kBatch) {
        float t[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) t[i] = k0 + i < a.K ? dxk[(size_t)(k0 + i) * a.n + q] : 0.f;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) g += t[i];
    }
    if (dz_out) dz_out[q] = g;
    if (failed) return;
    const float mq = a.beta1 * m[q] + (1.0f - a.beta1) * g;
    const float vq = a.beta2 * v[q] + (1.0f - a.beta2) * g * g;
    m[q] = mq;
    v[q] = vq;
    z[q] -= a.lr * (mq / a.corr1) / (sqrtf(vq / a.corr2) + a.eps);
}

__global__ void lane_shift_probe_kernel(int *out)
{
    const int t = threadIdx.x;
    out[t] = lane_shr1_i32(t, -1);
    out[64 + t] = lane_shl1_i32(t, -2);
}

}  // namespace sdtw
