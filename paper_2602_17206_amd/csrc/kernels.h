// HIP kernels of the Soft-DTW hot path for gfx950.  Included once by sdtw_api.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "device_core.h"
#include "layout.h"

namespace sdtw {

constexpr int kStatusState = 4;    // SDTW_ERR_STATE
constexpr int kStatusTimeout = 6;  // SDTW_ERR_TIMEOUT
constexpr int kBlkFloats = kBlk * kLdsStride;  // floats of one 32x32 block in LDS (padded rows)

// ---------------------------------------------------------------------------------------------
// Small utility kernels
// ---------------------------------------------------------------------------------------------
__global__ void fill_u64_kernel(unsigned long long *dst, size_t n, unsigned long long v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = v;
}

__global__ void fill_f32_kernel(float *dst, size_t n, float v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = v;
}

// Stamps the header at the start of a forward call.
__global__ void forward_begin_kernel(Params p)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        Header *h = p.hdr;
        h->magic = kMagic;
        h->B = p.B; h->N = p.N; h->M = p.M; h->D = p.D; h->mode = p.mode;
        h->gamma_bits = __float_as_uint(p.gamma);
        h->forward_done = 1;
        h->status = 0;
        h->abort_backward = 0;
        h->fwd_ticket = 0;
        h->bwd_ticket = 0;
    }
}

// Checks at the start of a backward call that the workspace holds the forward of this descriptor.
__global__ void backward_begin_kernel(Params p)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        Header *h = p.hdr;
        const bool ok = h->magic == kMagic && h->forward_done == 1 && h->B == p.B && h->N == p.N &&
                        h->M == p.M && h->D == p.D && h->mode == p.mode &&
                        h->gamma_bits == __float_as_uint(p.gamma);
        h->bwd_ticket = 0;
        if (ok) {
            h->abort_backward = 0;
        } else {
            h->magic = kMagic;  // make the status word meaningful even on an untouched buffer
            h->forward_done = 0;
            h->abort_backward = 1;
            h->status = kStatusState;
        }
    }
}

// ||row||^2 for `rows` rows of length D (Sec. 4.3: the squared norms are computed once).
// One wavefront per row, lanes stride over the features.
__global__ __launch_bounds__(256) void row_sqnorm_kernel(const float *__restrict__ v, float *__restrict__ out,
                                                        int64_t rows, int D)
{
    const int lane = threadIdx.x & 63;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t stride = (int64_t)gridDim.x * 4;
    for (; row < rows; row += stride) {
        const float *r = v + row * D;
        float acc = 0.f;
        for (int k = lane; k < D; k += 64) acc = fmaf(r[k], r[k], acc);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) out[row] = acc;
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
// Cost blocks into the LDS ring of a band.
// ring[(rb*2 + slot)][32 rows][kLdsStride]: rb = upper/lower 32 rows of the band, slot = cb & 1.
// ---------------------------------------------------------------------------------------------
template <bool FUSED>
__device__ __forceinline__ void produce_block(const Params &p, int b, int row0, int rb, int cb,
                                              float *ring, int lane)
{
    float *blk = ring + (rb * 2 + (cb & 1)) * kBlkFloats;
    const int i0 = row0 + rb * 32, j0 = cb * 32;
    if (FUSED) {
        float out[16];
        cost_block(p, p.x + b * p.x_stride, p.y + b * p.y_stride, p.xn + b * p.xn_stride,
                   p.yn + b * p.yn_stride, i0, j0, lane, out);
        const int col = lane & 31;
#pragma unroll
        for (int i = 0; i < 16; ++i) blk[acc_row(i, lane) * kLdsStride + col] = out[i];
    } else {
        const float *src = p.cost + (size_t)b * p.N * p.M;
        const int c4 = (lane & 7) * 4;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = (lane >> 3) + 8 * it;
            const int row = min(i0 + r, p.N - 1);
            const float *q = src + (size_t)row * p.M + j0 + c4;
            float4 v;
            if (p.vec_m && j0 + c4 + 3 < p.M) {
                v = *reinterpret_cast<const float4 *>(q);
            } else {
                v.x = (j0 + c4 + 0 < p.M) ? q[0] : 0.f;
                v.y = (j0 + c4 + 1 < p.M) ? q[1] : 0.f;
                v.z = (j0 + c4 + 2 < p.M) ? q[2] : 0.f;
                v.w = (j0 + c4 + 3 < p.M) ? q[3] : 0.f;
            }
            *reinterpret_cast<float4 *>(blk + r * kLdsStride + c4) = v;
        }
    }
}

// Waits until the 32 boundary values this macro-step needs have been written by the neighbouring
// band (they are initialised to kSentinel), and returns this lane's value.  The values are
// published with single 64-bit device-scope atomic stores, so every value validates itself and
// no flag or fence is needed.  A band gives up after p.spin_limit polls, records
// SDTW_ERR_TIMEOUT and never waits again (gave_up); other bands see the recorded status and stop
// waiting too, so a failure costs one time-out period in total, not one per wait.
__device__ __forceinline__ double wait_boundary(const Params &p, const unsigned long long *row, int jj,
                                                bool need, int lane, bool &gave_up)
{
    unsigned long long bits = 0x7FF0000000000000ull;  // +inf
    unsigned spins = 0;
    for (;;) {
        if (need) bits = __hip_atomic_load(row + jj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ok = !need || bits != kSentinel;
        if (__all(ok) || gave_up) break;
        ++spins;
        bool stop = spins > p.spin_limit;
        if (!stop && (spins & 255u) == 0)
            stop = __hip_atomic_load(&p.hdr->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == kStatusTimeout;
        if (stop) {
            if (lane == 0) atomicMax(&p.hdr->status, kStatusTimeout);
            gave_up = true;
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    return __longlong_as_double((long long)bits);
}

// ---------------------------------------------------------------------------------------------
// Forward DP (Sec. 2 Eq. 1-2, anti-diagonal order of Sec. 4.1).
// One wavefront = one band task (pair b, rows row0..row0+63).  Band tasks are handed out by an
// atomic ticket in band-major order, so a band only ever waits for a band with a smaller
// ticket, which is already running or done: the wait always ends.
// The table is written to HBM in step-major order R[b][band][s][lane] (one coalesced 512-byte
// store per step) and the band's last row goes to the boundary buffer for the next band.
// ---------------------------------------------------------------------------------------------
template <bool FUSED>
__global__ __launch_bounds__(64) void forward_dp_kernel(Params p, float *__restrict__ value)
{
    __shared__ __attribute__((aligned(16))) float ring[4 * kBlkFloats];
    __shared__ double edge[kBlk];

    const int lane = threadIdx.x;
    unsigned ticket = 0;
    if (lane == 0) ticket = atomicAdd(&p.hdr->fwd_ticket, 1u);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    const int k = ticket / (unsigned)p.B;
    const int b = ticket - k * p.B;
    if (k >= p.nbands) return;

    const int M = p.M;
    const int row0 = k * kBandRows, my_row = row0 + lane;
    const bool row_valid = my_row < p.N;
    const bool lower_rows = row0 + 32 < p.N;  // the band has rows in its second 32-row block
    const double INF = __builtin_inf();
    const float c2 = p.inv_gamma_log2e, g2 = p.gamma_ln2;

    bool gave_up = false;
    double left = INF;                                  // R[i][j-1]
    double diag = (k == 0 && lane == 0) ? 0.0 : INF;    // R[i-1][j-1]; R[0,0] = 0 in the paper's indexing
    const unsigned long long *brow_in = p.brow + ((size_t)b * p.nbands + (k > 0 ? k - 1 : 0)) * M;
    unsigned long long *brow_out = p.brow + ((size_t)b * p.nbands + k) * M;
    double *Rw = p.R + ((size_t)b * p.nbands + k) * (size_t)p.nmacro * kBlk * kBandRows;
    const bool emit_bottom = (k + 1 < p.nbands);
    const int jfin = (my_row == p.N - 1) ? M - 1 : -0x40000000;
    const float *my_ring = ring + ((lane >> 5) * 2) * kBlkFloats + (lane & 31) * kLdsStride;

    for (int sg = 0; sg < p.nmacro; ++sg) {
        // cost blocks that become live in this macro-step
        if (sg < p.ncb) produce_block<FUSED>(p, b, row0, 0, sg, ring, lane);
        if (sg >= 1 && sg - 1 < p.ncb && lower_rows) produce_block<FUSED>(p, b, row0, 1, sg - 1, ring, lane);

        // row above the band, columns 32*sg .. 32*sg+31
        double topv = INF;
        if (k > 0) {
            const int jj = sg * kBlk + lane;
            topv = wait_boundary(p, brow_in, jj, lane < kBlk && jj < M, lane, gave_up);
        }
        __syncthreads();

#pragma unroll
        for (int u = 0; u < kBlk; ++u) {
            const int s = sg * kBlk + u;
            const int j = s - lane;
            const double up = lane_shr1(left, read_lane(topv, u));  // R[i-1][j]
            const float dc = my_ring[((j >> 5) & 1) * kBlkFloats + (j & 31)];
            const bool active = row_valid && (unsigned)j < (unsigned)M;
            const double sm = softmin3(diag, up, left, c2, g2);
            const double cur = active ? sm + (double)dc : INF;
            Rw[(size_t)s * kBandRows + lane] = cur;
            if (j == jfin) {
                p.rfinal[b] = cur;
                value[b] = (float)cur;
            }
            if (lane == kBandRows - 1) edge[u] = cur;
            diag = up;
            left = cur;
        }
        __syncthreads();

        if (emit_bottom && lane < kBlk) {
            const int j = sg * kBlk + lane - (kBandRows - 1);
            if (j >= 0 && j < M)
                __hip_atomic_store(brow_out + j, (unsigned long long)__double_as_longlong(edge[lane]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Backward DP (Sec. 2 "Backward pass", Sec. 4.2).
//
// The paper carries Ebar = log E with
//   Ebar[i,j] = logsumexp(Ebar[i+1,j]+alpha, Ebar[i,j+1]+beta, Ebar[i+1,j+1]+delta),
//   alpha = (R[i+1,j] - R[i,j] - d[i+1,j])/gamma  (beta, delta alike).
// Substituting T[i,j] := R[N,M] - gamma*Ebar[i,j] - R[i,j] + d[i,j] turns this, term by term,
// into
//   T[i,j] = d[i,j] + softmin_gamma(T[i+1,j], T[i,j+1], T[i+1,j+1]),   T[N+1,M+1] := 0,
//   Ebar[i,j] = (R[N,M] - R[i,j] - (T[i,j] - d[i,j])) / gamma,
// the same log-space recurrence with the logarithm scaled by gamma.  It is still max-shifted
// log-sum-exp arithmetic (nothing can overflow for small gamma), it needs one cost value per cell
// instead of three, and the only large-magnitude subtraction, R[N,M] - R[i,j] - (T-d), happens once
// per cell in float64.  E = exp(Ebar) is applied per cell as soon as Ebar is known.
//
// Bands run bottom-up; lane t needs lane t+1's values, the band below supplies lane 63's.
// E leaves through LDS (in place of the consumed cost block) as row-major 32x32 blocks, with one
// flag byte per block saying whether any entry is non-zero.
// ---------------------------------------------------------------------------------------------
template <bool FUSED>
__global__ __launch_bounds__(64) void backward_dp_kernel(Params p)
{
    __shared__ __attribute__((aligned(16))) float ring[4 * kBlkFloats];
    __shared__ double edge[kBlk];

    const int lane = threadIdx.x;
    if (p.hdr->abort_backward) return;
    unsigned ticket = 0;
    if (lane == 0) ticket = atomicAdd(&p.hdr->bwd_ticket, 1u);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    const int kk = ticket / (unsigned)p.B;
    const int b = ticket - kk * p.B;
    if (kk >= p.nbands) return;
    const int k = p.nbands - 1 - kk;

    const int M = p.M;
    const int row0 = k * kBandRows, my_row = row0 + lane;
    const bool row_valid = my_row < p.N;
    const bool lower_rows = row0 + 32 < p.N;
    const double INF = __builtin_inf();
    const float c2 = p.inv_gamma_log2e, g2 = p.gamma_ln2;

    bool gave_up = false;
    double right = INF;  // T[i][j+1]
    double diag = INF;   // T[i+1][j+1]
    const int jcorner = (my_row == p.N - 1) ? M - 1 : -0x40000000;  // cell whose diagonal successor is T[N+1,M+1]=0
    const double Rfin = p.rfinal[b];
    const bool has_below = (k + 1 < p.nbands);
    const unsigned long long *brow_in = p.brow + ((size_t)b * p.nbands + (has_below ? k + 1 : k)) * M;
    unsigned long long *brow_out = p.brow + ((size_t)b * p.nbands + k) * M;
    const double *Rw = p.R + ((size_t)b * p.nbands + k) * (size_t)p.nmacro * kBlk * kBandRows;
    float *my_ring = ring + ((lane >> 5) * 2) * kBlkFloats + (lane & 31) * kLdsStride;
    float *Eb = p.E + (size_t)b * p.N * M;
    unsigned char *nzb = p.nz + (size_t)b * p.nrb * p.ncb;

    double Rcur[kBlk], Rnext[kBlk];
    const int sg0 = p.nmacro - 1;
#pragma unroll
    for (int u = 0; u < kBlk; ++u) Rcur[u] = Rw[((size_t)sg0 * kBlk + u) * kBandRows + lane];

    // blocks the first macro-step touches beyond the per-step rule below
    if (sg0 < p.ncb) produce_block<FUSED>(p, b, row0, 0, sg0, ring, lane);
    if (sg0 - 1 >= 0 && sg0 - 1 < p.ncb && lower_rows) produce_block<FUSED>(p, b, row0, 1, sg0 - 1, ring, lane);

    for (int sg = sg0; sg >= 0; --sg) {
        if (sg - 1 >= 0 && sg - 1 < p.ncb) produce_block<FUSED>(p, b, row0, 0, sg - 1, ring, lane);
        if (sg - 2 >= 0 && sg - 2 < p.ncb && lower_rows) produce_block<FUSED>(p, b, row0, 1, sg - 2, ring, lane);

        if (sg > 0) {
#pragma unroll
            for (int u = 0; u < kBlk; ++u) Rnext[u] = Rw[((size_t)(sg - 1) * kBlk + u) * kBandRows + lane];
        }

        // row below the band, columns 32*sg-63 .. 32*sg-32 (what lane 63 meets in this macro-step)
        double botv = INF;
        if (has_below) {
            const int jj = sg * kBlk + lane - (kBandRows - 1);
            botv = wait_boundary(p, brow_in, jj, lane < kBlk && jj >= 0 && jj < M, lane, gave_up);
        }
        __syncthreads();

#pragma unroll
        for (int u = kBlk - 1; u >= 0; --u) {
            const int s = sg * kBlk + u;
            const int j = s - lane;
            const double down = lane_shl1(right, read_lane(botv, u));  // T[i+1][j]
            float *cell = my_ring + ((j >> 5) & 1) * kBlkFloats + (j & 31);
            const float dc = *cell;
            const bool active = row_valid && (unsigned)j < (unsigned)M;
            const double dg = (j == jcorner) ? 0.0 : diag;
            const double tq = softmin3(dg, down, right, c2, g2);  // T[i][j] - d[i][j]
            const double cur = active ? tq + (double)dc : INF;
            const float ebar2 = (float)((Rfin - Rcur[u]) - tq) * c2;  // log2 E
            if (active) *cell = __builtin_amdgcn_exp2f(ebar2);
            if (lane == 0) edge[u] = cur;
            diag = down;
            right = cur;
        }
        __syncthreads();

        // first row of the band, columns 32*sg .. 32*sg+31, for the band above
        if (k > 0 && lane < kBlk) {
            const int j = sg * kBlk + lane;
            if (j < M)
                __hip_atomic_store(brow_out + j, (unsigned long long)__double_as_longlong(edge[lane]),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }

        // E blocks completed by this macro-step: (upper rows, cb = sg) and (lower rows, cb = sg-1)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int cb = sg - rb;
            if (cb < 0 || cb >= p.ncb || (rb == 1 && !lower_rows)) continue;
            const float *blk = ring + (rb * 2 + (cb & 1)) * kBlkFloats;
            const int c4 = (lane & 7) * 4, j0 = cb * kBlk;
            bool any = false;
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int r = (lane >> 3) + 8 * it;
                const int row = row0 + rb * 32 + r;
                const float4 v = *reinterpret_cast<const float4 *>(blk + r * kLdsStride + c4);
                if (row < p.N) {
                    float *q = Eb + (size_t)row * M + j0 + c4;
                    if (p.vec_m && j0 + c4 + 3 < M) {
                        *reinterpret_cast<float4 *>(q) = v;
                        any |= (v.x != 0.f) | (v.y != 0.f) | (v.z != 0.f) | (v.w != 0.f);
                    } else {
                        if (j0 + c4 + 0 < M) { q[0] = v.x; any |= v.x != 0.f; }
                        if (j0 + c4 + 1 < M) { q[1] = v.y; any |= v.y != 0.f; }
                        if (j0 + c4 + 2 < M) { q[2] = v.z; any |= v.z != 0.f; }
                        if (j0 + c4 + 3 < M) { q[3] = v.w; any |= v.w != 0.f; }
                    }
                }
            }
            const bool blk_any = __any(any);
            if (lane == 0) nzb[(size_t)(row0 / kBlk + rb) * p.ncb + cb] = blk_any ? 1 : 0;
        }
        __syncthreads();

#pragma unroll
        for (int u = 0; u < kBlk; ++u) Rcur[u] = Rnext[u];
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
    const float *own = side == 0 ? p.x + b * p.x_stride : p.y + b * p.y_stride;   // sequence of the output side
    const float *oth = side == 0 ? p.y + b * p.y_stride : p.x + b * p.x_stride;   // sequence reduced over
    out += (size_t)b * P * p.D;
    const int wr = w >> 1, wc = w & 1;

    if (p.hdr->abort_backward) {
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

    for (int q0 = 0; q0 < Q; q0 += kBlk) {
        // skip when both 32x32 E blocks of this chunk are all zero
        const int qb = q0 / kBlk, mb = m0 / kBlk;
        bool live;
        if (side == 0) {
            live = nzb[(size_t)mb * p.ncb + qb] != 0;
            if (mb + 1 < p.nrb) live |= nzb[(size_t)(mb + 1) * p.ncb + qb] != 0;
        } else {
            live = nzb[(size_t)qb * p.ncb + mb] != 0;
            if (mb + 1 < p.ncb) live |= nzb[(size_t)qb * p.ncb + mb + 1] != 0;
        }
        if (!live) continue;

        __syncthreads();  // previous chunk's reads are done
        // A tile, k-major: At[k][m]
        if (side == 0) {
            // E rows i = m0+m (64), columns j = q0+k (32): thread -> (m = tid/4 .. , 8 floats)
            for (int e = tid; e < 64 * 8; e += 256) {
                const int m = e >> 3, k4 = (e & 7) * 4;
                const int i = m0 + m;
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (i < p.N) {
                    const float *q = Eb + (size_t)i * p.M + q0 + k4;
                    if (p.vec_m && q0 + k4 + 3 < p.M) {
                        const float4 t = *reinterpret_cast<const float4 *>(q);
                        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c) if (q0 + k4 + c < p.M) v[c] = q[c];
                    }
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) At[(k4 + c) * kGradStride + m] = v[c];
            }
        } else {
            // E rows i = q0+k (32), columns j = m0+m (64)
            for (int e = tid; e < 32 * 16; e += 256) {
                const int k = e >> 4, m4 = (e & 15) * 4;
                const int i = q0 + k;
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i < p.N) {
                    const float *q = Eb + (size_t)i * p.M + m0 + m4;
                    if (p.vec_m && m0 + m4 + 3 < p.M) {
                        t = *reinterpret_cast<const float4 *>(q);
                    } else {
                        if (m0 + m4 + 0 < p.M) t.x = q[0];
                        if (m0 + m4 + 1 < p.M) t.y = q[1];
                        if (m0 + m4 + 2 < p.M) t.z = q[2];
                        if (m0 + m4 + 3 < p.M) t.w = q[3];
                    }
                }
                *reinterpret_cast<float4 *>(At + k * kGradStride + m4) = t;
            }
        }
        // B tile: Bt[k][n] = oth[q0+k][n0+n]
        for (int e = tid; e < 32 * 16; e += 256) {
            const int k = e >> 4, n4 = (e & 15) * 4;
            const int q = q0 + k;
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (q < Q) {
                const float *src = oth + (size_t)q * p.D + n0 + n4;
                if (p.vec_xy && n0 + n4 + 3 < p.D) {
                    t = *reinterpret_cast<const float4 *>(src);
                } else {
                    if (n0 + n4 + 0 < p.D) t.x = src[0];
                    if (n0 + n4 + 1 < p.D) t.y = src[1];
                    if (n0 + n4 + 2 < p.D) t.z = src[2];
                    if (n0 + n4 + 3 < p.D) t.w = src[3];
                }
            }
            *reinterpret_cast<float4 *>(Bt + k * kGradStride + n4) = t;
        }
        __syncthreads();

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
                out[(size_t)m * p.D + n] = scale * (own[(size_t)m * p.D + n] * tot - acc[i]);
            }
        }
    }
}

// Copies E to the caller's buffer (NaN when the backward call was refused).
__global__ void export_E_kernel(Params p, float *__restrict__ dst)
{
    const size_t n = (size_t)p.B * p.N * p.M;
    const bool bad = p.hdr->abort_backward != 0;
    const float qnan = __builtin_nanf("");
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = bad ? qnan : p.E[i];
}

// Un-skews the step-major DP table into row-major R[b][i][j] (test hook).
__global__ void export_R_kernel(Params p, double *__restrict__ dst)
{
    const size_t n = (size_t)p.B * p.N * p.M;
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t band_elems = (size_t)p.nmacro * kBlk * kBandRows;
    for (; e < n; e += stride) {
        const int j = (int)(e % p.M);
        const size_t bi = e / p.M;
        const int i = (int)(bi % p.N);
        const int b = (int)(bi / p.N);
        const int k = i / kBandRows, t = i % kBandRows;
        dst[e] = p.R[((size_t)b * p.nbands + k) * band_elems + (size_t)(j + t) * kBandRows + t];
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

__global__ void barycenter_update_kernel(AdamParams a, const float *__restrict__ dxk /*[K][n]*/,
                                         const float *__restrict__ values /*[K]*/, float *__restrict__ z,
                                         float *__restrict__ m, float *__restrict__ v,
                                         float *__restrict__ loss, float *__restrict__ dz_out)
{
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q == 0) {
        float L = 0.f;
        for (int k = 0; k < a.K; ++k) L += values[k];
        loss[0] = L;
    }
    if (q >= a.n) return;
    float g = 0.f;
    for (int k = 0; k < a.K; ++k) g += dxk[(size_t)k * a.n + q];
    if (dz_out) dz_out[q] = g;
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
