// Workspace layout and kernel parameter blocks shared by the host entry points and the kernels.
//
// The DP works on row bands of 64 rows (one row per wavefront lane).  A band sweeps the columns
// in "steps": at step s lane t owns cell (row0+t, s-t), so all 64 cells of a step lie on one
// anti-diagonal (Sec. 4.1: cells of an anti-diagonal are independent).  Steps are grouped in
// macro-steps of 32 because the cost arrives in 32x32 blocks.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace sdtw {

constexpr int kBandRows = 64;    // rows per band == lanes per wavefront
constexpr int kBlk = 32;         // edge of a cost block (one 32x32 MFMA tile)
constexpr uint64_t kSentinel = 0xFFFFFFFFFFFFFFFFull;  // "not written yet" in boundary rows
constexpr uint32_t kMagic = 0x53445457u;               // 'SDTW'
constexpr double kBig = 1e300;                         // stands for +inf in the DP tables and boundary rows
constexpr int32_t kNoWindow = 0x3FFFFFFF;              // Params::window when there is no band constraint
constexpr int kGuardBytes = 512;  // slack before/after regions that are read with clamped indices

// First 256 bytes of a workspace (device memory).
struct Header {
    uint32_t magic;
    int32_t B, N, M, D, mode;
    uint32_t gamma_bits;
    int32_t forward_done;  // set by the forward call, checked by the backward call
    int32_t status;        // device-side sdtw_status (0, STATE, TIMEOUT)
    int32_t abort_backward;
    uint32_t fwd_ticket;   // next band task of the forward sweep
    uint32_t bwd_ticket;   // next band task of the backward sweep
    int32_t two_sweep;     // the forward call also ran the reverse sweep
    int32_t window;        // band constraint |i-j| <= window the forward was run with (kNoWindow: none)
    uint64_t x_len_ptr, y_len_ptr;  // the length vectors the forward was run with (0: none)
    uint32_t pool_count;   // compact E: 32x32 blocks handed out so far (may run past the capacity)
    int32_t pool_overflow; // compact E: a block did not fit; the backward call redoes the gradients the slow way
    int32_t pieces;        // float16 pieces per operand element the forward was run with (Params::pieces)
    uint32_t pad[43];
};
static_assert(sizeof(Header) == 256, "header is 256 bytes");

struct Params;

struct Layout {
    int32_t B, N, M, D, mode;
    int32_t nbands;   // ceil(N/64)
    int32_t nmacro;   // macro-steps per band sweep: ceil((M+63)/32)
    int32_t nm_tab;   // macro-steps of table (R, Q, checkpoints) kept per band: nmacro, fewer under a band constraint
    int32_t nrb, ncb; // 32x32 block rows / columns: ceil(N/32), ceil(M/32)
    int64_t xn_count, yn_count;  // number of norm entries (1 sequence when the batch stride is 0)
    int32_t Dp;                  // D rounded up to 16, 32, 64 or 128: row length of the split-half operand copies (0: none)
    int32_t recompute;           // 1: checkpoints instead of the R table (large problems)
    int32_t two_sweep;           // 1: the forward call also runs the reverse sweep and stores its table Q
    int32_t compact_E;           // 1: E is kept as a pool of its non-zero 32x32 blocks, not as a dense tensor (see make_layout)
    int64_t pool_blocks;         // capacity of that pool
    size_t off_hdr, off_rfinal, off_xn, off_yn, off_xis, off_yis, off_xh, off_yh, off_brow, off_brow_b, off_R,
        off_Q, off_ckpt, off_cost, off_E, off_nz, off_idx, off_pool, off_rsum, off_csum, off_dyhi, off_pexp, off_self, total;
};

// With D <= 128 the workspace keeps a copy of x and y split into two float16 pieces per element
// (made by forward_prep_kernel) for the fp16 matrix cores; larger D computes the cost in float32
// straight from x and y.
constexpr int kMaxSplitD = 128;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// table steps kept per band (multiple of 32; without a band constraint all of the sweep's, >= M+63)
inline int64_t steps_of(const Layout &L) { return (int64_t)L.nm_tab * kBlk; }

// Under a band constraint |i-j| <= window a band only ever runs macro-steps between the first one of
// the band above it and the last one of the band below it (alone, or as either half of a chained
// pair): at most (2*window + 256)/32 + 3 of them.  Its tables hold that many, starting at the
// macro-step table_base() (device_core.h) returns.
inline int32_t table_macro_steps(int32_t nmacro, int32_t window)
{
    if (window >= kNoWindow) return nmacro;
    const int64_t need = (2 * (int64_t)window + 4 * kBandRows) / kBlk + 3;
    return need < nmacro ? (int32_t)need : nmacro;
}

// Large problems with long sequences keep the alignment matrix compactly (see make_layout): from this
// many cells per pair on, or whenever the caller asks for little memory.
constexpr int64_t kCompactCells = (int64_t)1 << 24;

inline Layout make_layout(int32_t B, int32_t N, int32_t M, int32_t D, int32_t mode, bool x_shared,
                          bool y_shared, bool recompute, bool two_sweep, int32_t window = kNoWindow,
                          int compact = 0 /* -1: never, 0: by size, 1: always (where the regime allows) */)
{
    Layout L{};
    L.B = B; L.N = N; L.M = M; L.D = D; L.mode = mode;
    L.nbands = (N + kBandRows - 1) / kBandRows;
    L.nmacro = (M + kBandRows - 1 + kBlk - 1) / kBlk;
    L.nm_tab = table_macro_steps(L.nmacro, window);
    L.nrb = (N + kBlk - 1) / kBlk;
    L.ncb = (M + kBlk - 1) / kBlk;
    L.xn_count = (int64_t)(x_shared ? 1 : B) * N;
    L.yn_count = (int64_t)(y_shared ? 1 : B) * M;
    size_t o = 0;
    L.off_hdr = o;      o += sizeof(Header);
    L.off_rfinal = o;   o = align_up(o + (size_t)B * sizeof(double), 256);
    L.off_xn = o;       o = align_up(o + (size_t)L.xn_count * sizeof(float), 256);
    L.off_yn = o;       o = align_up(o + (size_t)L.yn_count * sizeof(float), 256);
    L.Dp = D <= 16 ? 16 : (D <= 32 ? 32 : (D <= 64 ? 64 : (D <= kMaxSplitD ? 128 : 0)));
    L.off_xis = o;      o = align_up(o + (size_t)(L.Dp ? L.xn_count : 0) * sizeof(float), 256);
    L.off_yis = o;      o = align_up(o + (size_t)(L.Dp ? L.yn_count : 0) * sizeof(float), 256);
    L.off_xh = o;       o = align_up(o + (size_t)L.xn_count * L.Dp * 2 * sizeof(uint16_t), 256);
    L.off_yh = o;       o = align_up(o + (size_t)L.yn_count * L.Dp * 2 * sizeof(uint16_t), 256);
    // boundary rows: one row of M float64 per (pair, band)
    L.recompute = recompute ? 1 : 0;
    L.two_sweep = two_sweep ? 1 : 0;
    const size_t brow_bytes = (size_t)B * L.nbands * (size_t)M * sizeof(double);
    L.off_brow = o;     o = align_up(o + brow_bytes, 256);
    // the reverse sweep gets rows of its own when the forward's must survive (recomputation) or when
    // both sweeps run at the same time
    const bool own_rows = recompute || two_sweep;
    L.off_brow_b = own_rows ? o : L.off_brow;
    if (own_rows) o = align_up(o + brow_bytes, 256);
    // DP table in step-major order: [B][nbands][steps][64] float64 - or, with recomputation, only
    // the lane state (left, diagonal) at the start of every macro-step: [B][nbands][nmacro][2][64]
    const size_t table_bytes = (size_t)B * L.nbands * (size_t)steps_of(L) * kBandRows * sizeof(double);
    L.off_R = o;
    if (!recompute) o = align_up(o + table_bytes, 256);
    // table of the reverse sweep, same order as R
    L.off_Q = o;
    if (two_sweep) o = align_up(o + table_bytes, 256);
    L.off_ckpt = o;
    if (recompute) o = align_up(o + (size_t)B * L.nbands * (size_t)L.nm_tab * 2 * kBandRows * sizeof(double), 256);
    o += kGuardBytes;
    L.off_cost = o;
    if (mode == 0) o = align_up(o + (size_t)B * N * (size_t)M * sizeof(float), 256);
    o += kGuardBytes;
    // The alignment matrix E.  Dense, [B,N,M] float32 - or, for large problems with long sequences
    // (and split operand copies, D <= 128), compact: the reverse sweep stores only the 32x32 blocks that
    // hold a non-zero, into a pool of blocks handed out by an atomic counter, with an index
    // [B, N/32, M/32] that says where each block went (-1: all zero).  For the small gamma that long
    // alignments are run with, E is a few blocks wide around the alignment path: the pool has room for
    // 1/64 of all blocks, at least 2 (N/32 + M/32) per pair (a path crosses N/32 + M/32 - 1 of them).  When
    // the pool runs over, the backward call forms the gradients once more with a reverse sweep that
    // contracts every block of E into them on the spot (slow: that work then sits in the chain of
    // dependent steps; callers with long sequences AND dense E ask for the dense layout).  The sums of
    // that second sweep live where the pool was.
    const bool long_pairs = (int64_t)N * M >= kCompactCells;
    L.compact_E = (recompute && L.Dp > 0 && (compact > 0 || (compact == 0 && long_pairs))) ? 1 : 0;
    L.off_E = o;
    if (!L.compact_E) o = align_up(o + (size_t)B * N * (size_t)M * sizeof(float), 256);
    o += kGuardBytes;
    L.off_nz = o;       o = align_up(o + (size_t)B * L.nrb * (size_t)L.ncb, 256);
    L.off_idx = L.off_pool = L.off_rsum = L.off_csum = L.off_dyhi = L.off_pexp = L.off_self = o;
    L.pool_blocks = 0;
    if (L.compact_E) {
        L.off_self = o;  o += 1024;  // a copy of the kernel parameter block (Params::self)
        const int64_t all = (int64_t)B * L.nrb * L.ncb;
        L.pool_blocks = all / 64 > 2 * (int64_t)B * (L.nrb + L.ncb) ? all / 64 : 2 * (int64_t)B * (L.nrb + L.ncb);
        if (L.pool_blocks > all) L.pool_blocks = all;
        L.off_idx = o;  o = align_up(o + (size_t)all * sizeof(int32_t), 256);
        L.off_pool = o;
        const size_t pool_bytes = (size_t)L.pool_blocks * kBlk * kBlk * sizeof(float);
        // the second sweep's sums, in the same place: rsum [B,N], csum 2 x [B,M] words, gdy_hi [B,M,D], pair_exp [B]
        size_t q = o;
        L.off_rsum = q;  q = align_up(q + (size_t)B * N * sizeof(float), 256);
        L.off_csum = q;  q += 2 * align_up((size_t)B * M * sizeof(uint32_t), 256);
        L.off_dyhi = q;  q = align_up(q + (size_t)B * M * (size_t)D * sizeof(int32_t), 256);
        L.off_pexp = q;  q = align_up(q + (size_t)B * sizeof(int32_t), 256);
        o = align_up(o + (pool_bytes > q - o ? pool_bytes : q - o), 256);
    }
    L.total = o;
    return L;
}

// Everything a kernel needs; passed by value.
struct Params {
    int32_t B, N, M, D, mode;
    int32_t nbands, nmacro, nrb, ncb;
    int32_t nm_tab;         // macro-steps of table kept per band (see table_macro_steps)
    float gamma;
    double c2d;             // log2(e)/gamma: paper units -> table units
    double inv_c2d;         // gamma*ln(2): table units -> paper units
    int64_t x_stride, y_stride;    // batch strides of x, y (elements)
    int64_t xn_stride, yn_stride;  // batch strides of the norm vectors (0 when shared)
    int32_t vec_xy;                // 1: D%8==0 and x,y 16-byte aligned -> float4 operand loads
    int32_t vec_d4;                // 1: D%4==0 and x,y 16-byte aligned -> float4 loads of register operands
    int32_t vec_m;                 // 1: M%4==0 -> float4 loads/stores of cost and E rows
    uint32_t spin_limit;           // polls before a band gives up waiting
    const float *x, *y;
    const int32_t *x_len, *y_len;  // ragged batches: per-pair lengths (device), or nullptr
    int32_t window;                // only cells with |i-j| <= window belong to the grid (kNoWindow: all do)
    Header *hdr;
    double *rfinal;
    float *xn, *yn;
    int32_t Dp;                    // row length (halves) of the split operand copies, 0 if absent
    int32_t pieces;                // 2: x, y are float32, each element is two float16 pieces (three matrix-core products);
                                   // 1: x, y hold float16 / bfloat16 values (the *_half entry points): the first piece is
                                   //    the whole element, one product
    float *xis, *yis;              // per row: 1/scale used for the split copy (a power of two)
    uint16_t *xh, *yh;             // [rows][Dp/16][2 pieces][16] float16 bit patterns
    int64_t xh_stride, yh_stride;  // batch strides of the split copies (0 when shared)
    unsigned long long *brow;      // boundary rows of the forward sweep
    unsigned long long *brow_b;    // boundary rows of the backward sweep (rows of its own whenever a backward can follow)
    double *R;
    double *Q;                     // two_sweep: table of the reverse sweep (soft-minimum part), ordered like R
    double *ckpt;                  // large problems: forward lane state per macro-step instead of R
    int32_t two_sweep;
    float *cost;
    float *E;                      // alignment matrix, dense: in the workspace, or the caller's E_out where the workspace has none
    unsigned char *nz;
    // compact E (Layout::compact_E, no E_out wanted): block (rb, cb) of pair b is pool + 1024 * idx[...] floats,
    // row-major 32 x 32, if idx >= 0; pool_blocks = capacity
    float *pool;
    int32_t *idx;
    int64_t pool_blocks;
    // Reverse sweep that contracts E into the gradients itself (second sweep of a compact layout whose pool ran over):
    // gdx [B,N,D] / gdy [B,M,D] accumulate sum_j E_ij y_j / sum_i E_ij x_i (the caller's dx, dy buffers,
    // either may be null), rsum [B,N] / csum [B,M] the marginal sums of E; gradient_finish_kernel
    // turns them into dx, dy.
    // The y side is summed over all bands of a pair at once, in fixed point with integer atomics (exact
    // in any order): unit 2^(pair_exp[b] - fx_prec), low fx_lo_bits bits of every term into gdy (as
    // unsigned), the rest into gdy_hi; the column sums of E likewise (unit 2^-24) in csum_lo / csum_hi.
    float *gdx, *gdy;
    float *rsum;
    unsigned *csum_lo;
    int32_t *csum_hi, *gdy_hi;
    const int32_t *pair_exp;       // [B]: |x_b| < 2^pair_exp[b] (from the per-row scales of the split copies)
    int32_t fx_prec, fx_lo_bits;
    // This very block in device memory (written by second_sweep_prep_kernel): what the second sweep hands to
    // its out-of-line contraction routine by reference, so that the kernel need not keep a private copy.
    const Params *self;
};

}  // namespace sdtw
