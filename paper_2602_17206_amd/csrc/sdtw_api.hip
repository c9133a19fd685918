// C entry points of the Soft-DTW library (declared in include/sdtw.h): argument checks,
// workspace carving and kernel launches.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/sdtw.h"
#include "kernels.h"
#include "dp_kernels.h"
#include "layout.h"
#include "rate_probe.h"

namespace {

using namespace sdtw;

// Test hooks (process-wide; a change while another thread is inside a call of this library may be seen
// by part of that call only: set them between calls).
std::atomic<uint32_t> g_spin_limit{1u << 23};  // ~10 s of polling before a band gives up
std::atomic<int> g_force_slots{0};             // 0 = choose by problem size, 1, 2 or 4 = force that workgroup shape
std::atomic<long long> g_pool_blocks{-1};      // >= 0: capacity of the compact-E block pool (at most the layout's), to force an overflow

// Optional per-kernel timing (test/benchmark hook): when switched on, every kernel launch of the
// library is bracketed by two HIP events on the caller's stream.
struct ProfEntry { const char *name; hipEvent_t a, b; };
bool g_profile = false;
std::vector<ProfEntry> g_prof;

struct ProfScope {
    hipStream_t st;
    bool on;
    ProfScope(const char *name, hipStream_t s) : st(s), on(g_profile)
    {
        if (!on) return;
        ProfEntry e{name, nullptr, nullptr};
        if (hipEventCreate(&e.a) != hipSuccess || hipEventCreate(&e.b) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(e.a, st);
        g_prof.push_back(e);
    }
    ~ProfScope() { if (on) (void)hipEventRecord(g_prof.back().b, st); }
};

bool desc_ok(const sdtw_desc *d, int *why)
{
    *why = SDTW_ERR_INVALID_ARG;
    if (!d) return false;
    if (d->B < 1 || d->N < 1 || d->M < 1 || d->D < 1) return false;
    if (d->B > 32767) return false;
    if (!(d->gamma > 0.0f) || !std::isfinite(d->gamma)) return false;
    if (d->mode != SDTW_UNFUSED && d->mode != SDTW_FUSED) return false;
    if ((d->flags & ~(uint32_t)(SDTW_FLAG_VALUE_ONLY | SDTW_FLAG_MIN_MEMORY | SDTW_FLAG_DENSE_E)) != 0) return false;
    if ((d->flags & SDTW_FLAG_MIN_MEMORY) && (d->flags & SDTW_FLAG_DENSE_E)) return false;
    if (d->x_batch_stride != 0 && d->x_batch_stride != (int64_t)d->N * d->D) return false;
    if (d->y_batch_stride != 0 && d->y_batch_stride != (int64_t)d->M * d->D) return false;
    if ((int64_t)d->M + 128 > 0x3FFFFFFF || (int64_t)d->N + 128 > 0x3FFFFFFF) return false;
    // band constraint |i-j| <= bandwidth: the last cell (N-1, M-1) has to be inside it
    if (d->bandwidth < 0 || d->bandwidth >= kNoWindow) return false;
    if (d->bandwidth > 0 && std::abs(d->N - d->M) > d->bandwidth) return false;
    *why = SDTW_OK;
    return true;
}

// A band at least as wide as the grid constrains nothing: treated as no band at all.
int32_t effective_window(const sdtw_desc *d)
{
    return (d->bandwidth > 0 && d->bandwidth < std::max(d->N, d->M)) ? d->bandwidth : kNoWindow;
}

// Bands of one pair that have work at the same time.  Without a band constraint all of them; with
// |i-j| <= w a band runs (2w+129)/32 + 2 macro-steps and the band below it starts 5 macro-steps
// after it (its window begins 64 columns further right), so only a few overlap.
int64_t busy_bands(const sdtw_desc *d)
{
    const int64_t nbands = (d->N + kBandRows - 1) / kBandRows;
    const int32_t w = effective_window(d);
    if (w >= kNoWindow) return nbands;
    const int64_t run = (2 * (int64_t)w + 2 * kBandRows + 1) / kBlk + 2;
    return std::min<int64_t>(nbands, run / 5 + 2);
}

// Problems of up to about 1536 busy band tasks cannot fill the chip: they run one band per workgroup
// (measured: 19 % faster than the 4-band workgroups at 1536 tasks, equal at 2048, 40 % slower at 4096).
// (Under a band constraint the estimate of the busy bands is coarse; measured at B = 32, N = M = 8192
// and B = 128, N = M = 2048 the one-band workgroups win up to about 640.)
bool small_problem(const sdtw_desc *d)
{
    if (g_force_slots) return g_force_slots != 4;
    if (d->flags & SDTW_FLAG_MIN_MEMORY) return false;  // checkpoints instead of tables, no stored E
    return (int64_t)d->B * busy_bands(d) <= (effective_window(d) < kNoWindow ? 640 : 1536);
}

Layout layout_of(const sdtw_desc *d)
{
    const bool small = small_problem(d);
    const bool recompute = !small;  // the 4-band workgroups keep checkpoints instead of R (dp_recompute)
    const bool two_sweep = small && !(d->flags & SDTW_FLAG_VALUE_ONLY);
    const int compact = (d->flags & SDTW_FLAG_DENSE_E) ? -1 : ((d->flags & SDTW_FLAG_MIN_MEMORY) ? 1 : 0);
    return make_layout(d->B, d->N, d->M, d->D, d->mode, d->x_batch_stride == 0, d->y_batch_stride == 0, recompute,
                       two_sweep, effective_window(d), compact);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Params make_params(const sdtw_desc *d, const Layout &L, const float *x, const float *y, void *ws,
                   const int32_t *x_len = nullptr, const int32_t *y_len = nullptr, int pieces = 2)
{
    Params p{};
    p.pieces = pieces;
    p.x_len = x_len;
    p.y_len = y_len;
    p.window = effective_window(d);
    char *base = static_cast<char *>(ws);
    p.B = d->B; p.N = d->N; p.M = d->M; p.D = d->D; p.mode = d->mode;
    p.nbands = L.nbands; p.nmacro = L.nmacro; p.nrb = L.nrb; p.ncb = L.ncb;
    p.nm_tab = L.nm_tab;
    p.gamma = d->gamma;
    p.c2d = 1.4426950408889634 / (double)d->gamma;
    p.inv_c2d = 0.6931471805599453 * (double)d->gamma;
    p.x_stride = d->x_batch_stride; p.y_stride = d->y_batch_stride;
    p.xn_stride = d->x_batch_stride == 0 ? 0 : d->N;
    p.yn_stride = d->y_batch_stride == 0 ? 0 : d->M;
    p.vec_xy = (d->D % 8 == 0) && aligned16(x) && aligned16(y) && (d->x_batch_stride % 4 == 0) &&
               (d->y_batch_stride % 4 == 0);
    p.vec_d4 = (d->D % 4 == 0) && aligned16(x) && aligned16(y) && (d->x_batch_stride % 4 == 0) &&
               (d->y_batch_stride % 4 == 0);
    p.vec_m = (d->M % 4 == 0);
    p.spin_limit = g_spin_limit;
    p.x = x; p.y = y;
    p.hdr = reinterpret_cast<Header *>(base + L.off_hdr);
    p.rfinal = reinterpret_cast<double *>(base + L.off_rfinal);
    p.xn = reinterpret_cast<float *>(base + L.off_xn);
    p.yn = reinterpret_cast<float *>(base + L.off_yn);
    p.Dp = L.Dp;
    p.xis = reinterpret_cast<float *>(base + L.off_xis);
    p.yis = reinterpret_cast<float *>(base + L.off_yis);
    p.xh = reinterpret_cast<uint16_t *>(base + L.off_xh);
    p.yh = reinterpret_cast<uint16_t *>(base + L.off_yh);
    p.xh_stride = d->x_batch_stride == 0 ? 0 : (int64_t)d->N * L.Dp * 2;
    p.yh_stride = d->y_batch_stride == 0 ? 0 : (int64_t)d->M * L.Dp * 2;
    p.brow = reinterpret_cast<unsigned long long *>(base + L.off_brow);
    p.brow_b = reinterpret_cast<unsigned long long *>(base + L.off_brow_b);
    p.R = reinterpret_cast<double *>(base + L.off_R);
    p.Q = reinterpret_cast<double *>(base + L.off_Q);
    p.two_sweep = L.two_sweep;
    p.ckpt = reinterpret_cast<double *>(base + L.off_ckpt);
    p.cost = reinterpret_cast<float *>(base + L.off_cost);
    p.E = L.compact_E ? nullptr : reinterpret_cast<float *>(base + L.off_E);  // (compact: the caller's E_out, if any)
    p.nz = reinterpret_cast<unsigned char *>(base + L.off_nz);
    p.pool = nullptr;  // (compact E: set by the backward call that uses the pool)
    p.idx = nullptr;
    p.pool_blocks = 0;
    // (the accumulators of a reverse sweep that forms the gradients itself: set by that backward call)
    p.gdx = p.gdy = p.rsum = nullptr;
    p.csum_lo = nullptr;
    p.csum_hi = p.gdy_hi = nullptr;
    p.pair_exp = nullptr;
    p.fx_prec = p.fx_lo_bits = 0;
    p.self = nullptr;
    return p;
}

// Fused DP kernel variant: number of 16-feature groups of the split-half operands (D <= 16, 32,
// 64, 128), or 0 for the any-D kernel that computes the cost in float32 straight from x and y.
int fused_variant(int D)
{
    if (D <= 16) return 1;
    if (D <= 32) return 2;
    if (D <= 64) return 4;
    if (D <= 128) return 8;
    return 0;
}

// Launches the DP kernels in the workgroup shape that suits the problem.  Up to about 1536 band tasks
// cannot fill the chip: each band gets a small workgroup of its own (consumer and producers on
// different SIMDs), and the forward call runs the reverse sweep in the same launch (FWD, unless
// only the value is wanted); its backward call launches no DP kernel.  Larger problems use 4-band
// workgroups in which the producer and the consumer of a band share a SIMD, forward sweep in the
// forward call, reverse sweep in the backward call.
// grad: the reverse sweep that contracts E into the gradients itself (second sweep of a compact layout)
template <bool FWD, int KCH>
void launch_dp_kch(const sdtw_desc *d, const Layout &L, const Params &p, float *value, hipStream_t st, [[maybe_unused]] bool grad)
{
    constexpr int NP = KCH > 0 ? 2 : 1;
    if (small_problem(d)) {
        // Pairs of consecutive bands share a workgroup (the hand-over between them stays in LDS)
        // when there are at least two bands and the producers are light: in the chained shape the
        // producers of a band share one SIMD, which the D = 128 matrix-core producers fill
        // (measured at N = M = 256: 57 us chained against 54 us, but 50 us against 53 us unfused).
        // It also wants a compute unit per workgroup: two chained workgroups on one compute unit put
        // two consumers on one SIMD (measured at N = M = 1024, B = 32: 5 % slower than unchained).
        const bool light = d->mode == SDTW_UNFUSED || d->D <= 64;
        const bool roomy = (int64_t)d->B * ((busy_bands(d) + 1) / 2) * (L.two_sweep ? 2 : 1) <= 256;
        // (under a band constraint the chain of band hops is all there is: chaining pays there too, 3-4 %)
        const bool chained = g_force_slots ? g_force_slots == 2 : (L.nbands >= 2 && (light || effective_window(d) < kNoWindow) && roomy);
        if constexpr (FWD) {
            if (chained) {
                const unsigned tasks = (unsigned)d->B * (unsigned)((L.nbands + 1) / 2);
                if (L.two_sweep)
                    both_sweeps_kernel<KCH, 2, NP><<<2 * tasks, wg_threads(2, NP), 0, st>>>(p, value);
                else
                    forward_dp_kernel<KCH, 2, NP><<<tasks, wg_threads(2, NP), 0, st>>>(p, value);
            } else {
                const unsigned tasks = (unsigned)d->B * (unsigned)L.nbands;
                // about four workgroups per compute unit: the wavefronts share SIMDs anyway, and one
                // producer per band (two wavefronts per workgroup instead of three) leaves the consumers
                // more of them (3 % at N = M = 1024, B = 32)
                if (L.two_sweep && KCH > 0 && 2 * tasks > 900)
                    both_sweeps_kernel<KCH, 1, 1><<<2 * tasks, wg_threads(1, 1), 0, st>>>(p, value);
                else if (L.two_sweep)
                    both_sweeps_kernel<KCH, 1, NP><<<2 * tasks, wg_threads(1, NP), 0, st>>>(p, value);
                else
                    forward_dp_kernel<KCH, 1, NP><<<tasks, wg_threads(1, NP), 0, st>>>(p, value);
            }
        }
    } else {
        const unsigned tasks = (unsigned)((d->B + 3) / 4) * (unsigned)L.nbands;
        // The forward splits the cost blocks over two producers per band (register budget 168 per
        // wavefront); the recomputing backward consumer needs more registers than that, and its
        // long macro-steps leave a single producer enough time.
        if constexpr (FWD)
            forward_dp_kernel<KCH, 4, NP><<<tasks, wg_threads(4, NP), 0, st>>>(p, value);
        else if constexpr (KCH != 0) {
            if (grad)
                backward_dp_kernel<KCH, 4, 1, true><<<tasks, wg_threads(4, 1), 0, st>>>(p);
            else
                backward_dp_kernel<KCH, 4, 1><<<tasks, wg_threads(4, 1), 0, st>>>(p);
        } else {
            backward_dp_kernel<KCH, 4, 1><<<tasks, wg_threads(4, 1), 0, st>>>(p);  // D > 128: no split copies, E is stored
        }
    }
}

template <bool FWD>
void launch_dp(const sdtw_desc *d, const Layout &L, const Params &p, float *value, hipStream_t st, bool grad = false)
{
    if (d->mode == SDTW_UNFUSED) return launch_dp_kch<FWD, -1>(d, L, p, value, st, grad);
    switch (fused_variant(d->D)) {
        case 1: return launch_dp_kch<FWD, 1>(d, L, p, value, st, grad);
        case 2: return launch_dp_kch<FWD, 2>(d, L, p, value, st, grad);
        case 4: return launch_dp_kch<FWD, 4>(d, L, p, value, st, grad);
        case 8: return launch_dp_kch<FWD, 8>(d, L, p, value, st, grad);
        default: return launch_dp_kch<FWD, 0>(d, L, p, value, st, grad);
    }
}

int check_ws(const void *ws, size_t bytes, size_t need)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || bytes < need) return SDTW_ERR_WORKSPACE;
    return SDTW_OK;
}

inline int hip_ok() { return hipGetLastError() == hipSuccess ? SDTW_OK : SDTW_ERR_HIP; }

unsigned fill_grid(size_t n) { size_t g = (n + 255) / 256; return (unsigned)(g < 1 ? 1 : (g > 4096 ? 4096 : g)); }

// Blocks for a prep kernel: enough for the boundary fill (one element per thread) and for the row
// norms (a block takes four rows at a time, four times over), capped.
unsigned prep_grid(const Params &p, int64_t norm_rows)
{
    const size_t fill = ((size_t)p.B * p.nbands * p.M + 255) / 256;
    const size_t rows = (size_t)(norm_rows + 15) / 16;
    const size_t g = fill > rows ? fill : rows;
    return (unsigned)(g < 1 ? 1 : (g > 8192 ? 8192 : g));
}

int forward_impl(const sdtw_desc *d, const float *x, const float *y, float *value, void *ws, hipStream_t st,
                 const int32_t *x_len = nullptr, const int32_t *y_len = nullptr, int pieces = 2)
{
    (void)hipGetLastError();  // what an earlier, unrelated call left behind is not this call's error
    const Layout L = layout_of(d);
    const Params p = make_params(d, L, x, y, ws, x_len, y_len, pieces);
    // Unfused mode, small problems: the start of the call is folded into the cost-tensor kernel (one
    // launch instead of two).  Not with a band constraint or length vectors (tiles outside them are
    // skipped), not without 16-byte rows, and only where the tiles are few (fewer than 512 of 128 x 128):
    // with more, splitting the rows again in every tile costs more than the launch (measured at
    // N = M = 1024, B = 32: 89 us against 19 + 65).
    const size_t tiles128 = (size_t)((d->M + 127) / 128) * ((d->N + 127) / 128) * d->B;
    const bool folded = d->mode == SDTW_UNFUSED && L.Dp > 0 && p.vec_d4 && p.window >= kNoWindow && !x_len && !y_len &&
                        tiles128 < 512;
    if (!folded) {
        ProfScope ps("forward_prep", st);
        forward_prep_kernel<<<prep_grid(p, L.xn_count + L.yn_count), 256, 0, st>>>(p, L.xn_count, L.yn_count);
    }
    if (d->mode == SDTW_UNFUSED) {
        ProfScope ps("cost_tensor", st);
        // 128 x 128 tiles, or 128 x 64 when those would leave most of the chip idle
        const bool narrow = tiles128 < 512;
        dim3 gh(narrow ? (d->M + 63) / 64 : (d->M + 127) / 128, (d->N + 127) / 128, d->B);
        auto launch = [&](auto kg) {
            constexpr int KG = decltype(kg)::value;
            if (folded)
                cost_tensor_prep_kernel<KG, 2><<<gh, 256, 0, st>>>(p);
            else if (narrow)
                cost_tensor_half_kernel<KG, 2><<<gh, 256, 0, st>>>(p);
            else
                cost_tensor_half_kernel<KG, 4><<<gh, 256, 0, st>>>(p);
        };
        switch (fused_variant(d->D)) {
            case 1: launch(std::integral_constant<int, 1>{}); break;
            case 2: launch(std::integral_constant<int, 2>{}); break;
            case 4: launch(std::integral_constant<int, 4>{}); break;
            case 8: launch(std::integral_constant<int, 8>{}); break;
            default: {
                dim3 g((d->M + 63) / 64, (d->N + 63) / 64, d->B);
                cost_tensor_kernel<<<g, 256, 0, st>>>(p);
            }
        }
    }
    {
        const bool unf = d->mode == SDTW_UNFUSED;
        ProfScope ps(L.two_sweep ? (unf ? "both_sweeps_unfused" : "both_sweeps_fused")
                                 : (unf ? "forward_dp_unfused" : "forward_dp_fused"), st);
        launch_dp<true>(d, L, p, value, st);
    }
    return hip_ok();
}

int backward_impl(const sdtw_desc *d, const float *x, const float *y, const float *grad_value, float *dx,
                  float *dy, float *E_out, void *ws, hipStream_t st, const int32_t *x_len = nullptr,
                  const int32_t *y_len = nullptr, int pieces = 2)
{
    (void)hipGetLastError();  // see forward_impl
    const Layout L = layout_of(d);
    Params p = make_params(d, L, x, y, ws, x_len, y_len, pieces);
    // Compact E (large problems with long sequences, or on request): the reverse sweep leaves only the
    // non-zero 32x32 blocks of E, in a pool, and the gradient kernel reads them through the block index.
    // If the pool was too small (device-side flag) the kernels after it - otherwise no-ops - form the
    // gradients once more with a reverse sweep that contracts E into them on the spot.  With E_out the
    // blocks go to the caller's dense memory instead and everything is as for the dense layout.
    const bool compact = L.compact_E && E_out == nullptr;
    if (L.compact_E && E_out != nullptr) p.E = E_out;
    if (compact) {
        char *base = static_cast<char *>(ws);
        p.pool = reinterpret_cast<float *>(base + L.off_pool);
        p.idx = reinterpret_cast<int32_t *>(base + L.off_idx);
        const long long forced = g_pool_blocks;
        p.pool_blocks = forced >= 0 ? std::min<long long>(forced, L.pool_blocks) : L.pool_blocks;
        p.gdx = dx;
        p.gdy = dy;
        p.rsum = reinterpret_cast<float *>(base + L.off_rsum);
        p.csum_lo = reinterpret_cast<unsigned *>(base + L.off_csum);
        p.csum_hi = reinterpret_cast<int32_t *>(base + L.off_csum + align_up((size_t)d->B * d->M * sizeof(uint32_t), 256));
        p.gdy_hi = reinterpret_cast<int32_t *>(base + L.off_dyhi);
        p.pair_exp = reinterpret_cast<const int32_t *>(base + L.off_pexp);
        p.self = reinterpret_cast<const Params *>(base + L.off_self);
        // Fixed-point format of the second sweep's y-side sums: a column receives at most two terms per
        // band (one per 32-row block), each below 2^(prec + 6) units.  With nb bits for their number, the
        // low word takes lo_bits = 32 - nb bits of every term and the high word the other
        // prec + 6 - lo_bits, which have to fit 31 bits nb times over: prec <= 57 - 2 nb (26 is plenty).
        int nb = 1;
        while ((1ll << nb) < 2ll * L.nbands + 1) ++nb;
        p.fx_lo_bits = 32 - nb;
        p.fx_prec = std::min(26, 57 - 2 * nb);
    }
    if (L.two_sweep) {
        // both tables are there: combine them (the kernel checks the workspace itself)
        ProfScope ps("alignment", st);
        // runs of 32-column blocks per band: whole bands when there are at least 512 of them,
        // shorter runs otherwise (more wavefronts; the two macro-steps past a run's end are re-read)
        const int64_t bands = (int64_t)d->B * L.nbands;
        const int nseg = (int)std::max<int64_t>(1, std::min<int64_t>(L.ncb, (512 + bands - 1) / bands));
        const int seg_blocks = (L.ncb + nseg - 1) / nseg;
        dim3 g((L.ncb + seg_blocks - 1) / seg_blocks, L.nbands, d->B);
        if (L.ncb + 2 <= kAlignRowMacro)  // short rows: a block row's E fits in LDS, one workgroup for each
            alignment_row_kernel<kAlignRowMacro, 8><<<dim3(2, L.nbands, d->B), 512, 0, st>>>(p);
        else if (L.ncb >= 16)
            alignment_kernel<true><<<g, 64, 0, st>>>(p, seg_blocks);
        else
            alignment_kernel<false><<<g, 64, 0, st>>>(p, seg_blocks);
    } else {
        {
            ProfScope ps("backward_prep", st);
            backward_prep_kernel<<<prep_grid(p, 0), 256, 0, st>>>(p);
        }
        {
            ProfScope ps(d->mode == SDTW_UNFUSED ? "backward_dp_unfused" : "backward_dp_fused", st);
            launch_dp<false>(d, L, p, nullptr, st);
        }
    }
    if (dx || dy) {
        const int P = std::max(dx ? d->N : 0, dy ? d->M : 0);
        dim3 g((P + 63) / 64, (d->D + 63) / 64, 2 * d->B);
        ProfScope ps("input_grad", st);
        if (L.Dp > 0)
            input_grad_half_kernel<<<g, 256, 0, st>>>(p, grad_value, dx, dy);
        else
            input_grad_kernel<<<g, 256, 0, st>>>(p, grad_value, dx, dy);
    }
    if (E_out) {
        const size_t n = (size_t)d->B * d->N * d->M;
        if (L.compact_E)
            complete_E_kernel<<<fill_grid(n), 256, 0, st>>>(p);  // the sweep wrote the non-zero blocks into E_out itself
        else
            export_E_kernel<<<fill_grid(n), 256, 0, st>>>(p, E_out);
    }
    if (compact && (dx || dy)) {
        // only if the pool ran over (each of these kernels looks at the flag first)
        ProfScope ps("second_sweep", st);
        if (dy) pair_exponent_kernel<<<d->B, 256, 0, st>>>(p, reinterpret_cast<int32_t *>(static_cast<char *>(ws) + L.off_pexp));
        second_sweep_prep_kernel<<<prep_grid(p, 0), 256, 0, st>>>(p);
        launch_dp<false>(d, L, p, nullptr, st, true);
        const bool vec = (d->D % 4 == 0) && aligned16(x) && aligned16(y) && (!dx || aligned16(dx)) && (!dy || aligned16(dy));
        const size_t n = (size_t)d->B * ((size_t)d->N + d->M) * d->D / (vec ? 4 : 1);
        if (vec)
            gradient_finish_kernel<4><<<fill_grid(n), 256, 0, st>>>(p, grad_value);
        else
            gradient_finish_kernel<1><<<fill_grid(n), 256, 0, st>>>(p, grad_value);
    }
    return hip_ok();
}

bool bary_ok(const sdtw_bary_desc *d)
{
    if (!d) return false;
    if (d->K < 1 || d->Lz < 1 || d->Lx < 1 || d->D < 1 || d->step < 1 || d->K > 32767) return false;
    if (!(d->gamma > 0.0f) || !std::isfinite(d->gamma)) return false;
    if (d->mode != SDTW_UNFUSED && d->mode != SDTW_FUSED) return false;
    if (!(d->lr > 0.0f) || !std::isfinite(d->lr)) return false;
    if (!(d->beta1 >= 0.0f && d->beta1 < 1.0f) || !(d->beta2 >= 0.0f && d->beta2 < 1.0f)) return false;
    if (!(d->eps > 0.0f) || !std::isfinite(d->eps)) return false;
    if ((d->flags & ~(uint32_t)SDTW_FLAG_MIN_MEMORY) != 0) return false;
    return true;
}

sdtw_desc bary_pair_desc(const sdtw_bary_desc *d)
{
    sdtw_desc s{};
    s.B = d->K; s.N = d->Lz; s.M = d->Lx; s.D = d->D;
    s.gamma = d->gamma; s.mode = d->mode;
    s.x_batch_stride = 0;
    s.y_batch_stride = (int64_t)d->Lx * d->D;
    s.bandwidth = 0; s.flags = d->flags & SDTW_FLAG_MIN_MEMORY;
    return s;
}

struct BaryLayout { size_t off_values, off_dx, off_pair_ws, total; };

BaryLayout bary_layout(const sdtw_bary_desc *d)
{
    BaryLayout L{};
    size_t o = 0;
    // the pair workspace comes first so that its header (status word) sits at offset 0
    L.off_pair_ws = o;
    const sdtw_desc s = bary_pair_desc(d);
    o = align_up(o + layout_of(&s).total, 256);
    L.off_values = o; o = align_up(o + (size_t)d->K * sizeof(float), 256);
    L.off_dx = o;     o = align_up(o + (size_t)d->K * d->Lz * (size_t)d->D * sizeof(float), 256);
    L.total = o;
    return L;
}

// Normalised Soft-DTW: the three plain problems and where their workspaces sit.
struct NormPlan {
    sdtw_desc xy, xx, yy;
    bool x_shared, y_shared;
    size_t off_xy, off_xx, off_yy, off_vals, off_gx, off_gy, total;
    // One batch of 3B pairs instead of three passes: equal lengths, nothing shared, and small enough
    // that one pass leaves the chip idle (and the host, at about 5 us per launch, would otherwise be
    // what the three passes wait for).  The operands are gathered into xs, ys; dxs, dys take the
    // batch's gradients.  (all's workspace comes first: its header carries the status word.)
    bool batched;
    sdtw_desc all;
    size_t off_all, off_xs, off_ys, off_dxs, off_dys;
};

NormPlan norm_plan(const sdtw_desc *d)
{
    NormPlan P{};
    P.x_shared = d->x_batch_stride == 0;
    P.y_shared = d->y_batch_stride == 0;
    P.all = *d;
    P.all.B = 3 * d->B;
    P.all.x_batch_stride = (int64_t)d->N * d->D;
    P.all.y_batch_stride = (int64_t)d->M * d->D;
    P.batched = d->N == d->M && !P.x_shared && !P.y_shared && (int64_t)d->B * 3 <= 0x7fffffff / 4 && small_problem(&P.all);
    if (P.batched) {
        const size_t seq = 3 * (size_t)d->B * d->N * (size_t)d->D * sizeof(float);
        size_t o = 0;
        P.off_all = o; o = align_up(o + layout_of(&P.all).total, 256);
        P.off_xs = o; o = align_up(o + seq, 256);
        P.off_ys = o; o = align_up(o + seq, 256);
        P.off_dxs = o; o = align_up(o + seq, 256);
        P.off_dys = o; o = align_up(o + seq, 256);
        P.off_vals = o; o = align_up(o + 3 * (size_t)d->B * sizeof(float), 256);
        P.total = o;
        return P;
    }
    P.xy = *d;
    P.xx = *d;
    P.xx.B = P.x_shared ? 1 : d->B;
    P.xx.M = d->N;
    P.xx.y_batch_stride = d->x_batch_stride;
    P.yy = *d;
    P.yy.B = P.y_shared ? 1 : d->B;
    P.yy.N = d->M;
    P.yy.x_batch_stride = d->y_batch_stride;
    size_t o = 0;
    P.off_xy = o; o = align_up(o + layout_of(&P.xy).total, 256);  // first: its header carries the status word
    P.off_xx = o; o = align_up(o + layout_of(&P.xx).total, 256);
    P.off_yy = o; o = align_up(o + layout_of(&P.yy).total, 256);
    P.off_vals = o; o = align_up(o + 3 * (size_t)d->B * sizeof(float), 256);
    P.off_gx = o; o = align_up(o + (size_t)P.xx.B * d->N * (size_t)d->D * sizeof(float), 256);
    P.off_gy = o; o = align_up(o + (size_t)P.yy.B * d->M * (size_t)d->D * sizeof(float), 256);
    P.total = o;
    return P;
}

// Scratch of sdtw_forward_static_scratch: the workspace of a value-only forward, held by every GPU the
// library runs on until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the kernels get the address that call returned for the current device.
constexpr size_t kStaticScratchBytes = SDTW_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;

// Device address of `scratch` on the current device, looked up once per device.
void *static_scratch_ptr()
{
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (ptrs[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        ptrs[dev] = ptr;
    }
    return ptrs[dev];
}

}  // namespace

extern "C" {

int sdtw_version(void) { return 100; }

const char *sdtw_status_string(int status)
{
    switch (status) {
        case SDTW_OK: return "ok";
        case SDTW_ERR_INVALID_ARG: return "invalid argument";
        case SDTW_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SDTW_ERR_UNSUPPORTED: return "unsupported option (normalised Soft-DTW takes no bandwidth)";
        case SDTW_ERR_STATE: return "backward called on a workspace without a matching forward";
        case SDTW_ERR_HIP: return "HIP runtime error";
        case SDTW_ERR_TIMEOUT: return "a band gave up waiting for its neighbour";
        default: return "unknown status";
    }
}

size_t sdtw_workspace_bytes(const sdtw_desc *desc)
{
    int why;
    if (!desc_ok(desc, &why)) return 0;
    return layout_of(desc).total;
}

int sdtw_forward(const sdtw_desc *desc, const float *x, const float *y, float *value, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y || !value) return SDTW_ERR_INVALID_ARG;
    if (int rc = check_ws(workspace, workspace_bytes, layout_of(desc).total)) return rc;
    return forward_impl(desc, x, y, value, workspace, static_cast<hipStream_t>(stream));
}

int sdtw_forward_static_scratch(const sdtw_desc *desc, const float *x, const float *y, float *value, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y || !value) return SDTW_ERR_INVALID_ARG;
    sdtw_desc d = *desc;
    d.flags |= SDTW_FLAG_VALUE_ONLY;  // no backward call can follow: the scratch belongs to the next call
    if (layout_of(&d).total > kStaticScratchBytes) return SDTW_ERR_WORKSPACE;
    void *ws = static_scratch_ptr();
    if (ws == nullptr) return SDTW_ERR_HIP;
    // (the start of the forward - forward_prep_kernel or cost_tensor_prep_kernel - stamps the header,
    // resets the tickets and refills the boundary rows: nothing of the last call's contents is read)
    return forward_impl(&d, x, y, value, ws, static_cast<hipStream_t>(stream));
}

int sdtw_backward(const sdtw_desc *desc, const float *x, const float *y, const float *grad_value, float *dx,
                  float *dy, float *E_out, void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y) return SDTW_ERR_INVALID_ARG;
    if (desc->flags & SDTW_FLAG_VALUE_ONLY) return SDTW_ERR_STATE;
    if (int rc = check_ws(workspace, workspace_bytes, layout_of(desc).total)) return rc;
    return backward_impl(desc, x, y, grad_value, dx, dy, E_out, workspace, static_cast<hipStream_t>(stream));
}

int sdtw_forward_ragged(const sdtw_desc *desc, const float *x, const float *y, const int32_t *x_len,
                        const int32_t *y_len, float *value, void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y || !value) return SDTW_ERR_INVALID_ARG;
    if (int rc = check_ws(workspace, workspace_bytes, layout_of(desc).total)) return rc;
    return forward_impl(desc, x, y, value, workspace, static_cast<hipStream_t>(stream), x_len, y_len);
}

int sdtw_backward_ragged(const sdtw_desc *desc, const float *x, const float *y, const int32_t *x_len,
                         const int32_t *y_len, const float *grad_value, float *dx, float *dy, float *E_out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y) return SDTW_ERR_INVALID_ARG;
    if (desc->flags & SDTW_FLAG_VALUE_ONLY) return SDTW_ERR_STATE;
    if (int rc = check_ws(workspace, workspace_bytes, layout_of(desc).total)) return rc;
    return backward_impl(desc, x, y, grad_value, dx, dy, E_out, workspace, static_cast<hipStream_t>(stream), x_len,
                         y_len);
}

// Reduced-precision inputs: the plain workspace first (its header carries the status word), then the
// float32 copies of x and y.
struct HalfLayout { size_t off_x, off_y, total; int64_t nx, ny; };

static HalfLayout half_layout(const sdtw_desc *d)
{
    HalfLayout H{};
    H.nx = (int64_t)(d->x_batch_stride == 0 ? 1 : d->B) * d->N * d->D;
    H.ny = (int64_t)(d->y_batch_stride == 0 ? 1 : d->B) * d->M * d->D;
    size_t o = align_up(layout_of(d).total, 256);
    H.off_x = o; o = align_up(o + (size_t)H.nx * sizeof(float), 256);
    H.off_y = o; o = align_up(o + (size_t)H.ny * sizeof(float), 256);
    H.total = o;
    return H;
}

size_t sdtw_half_workspace_bytes(const sdtw_desc *desc)
{
    int why;
    if (!desc_ok(desc, &why)) return 0;
    return half_layout(desc).total;
}

int sdtw_forward_half(const sdtw_desc *desc, const void *x, const void *y, int input_type, float *value,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!x || !y || !value) return SDTW_ERR_INVALID_ARG;
    if (input_type != SDTW_INPUT_F16 && input_type != SDTW_INPUT_BF16) return SDTW_ERR_INVALID_ARG;
    const HalfLayout H = half_layout(desc);
    if (int rc = check_ws(workspace, workspace_bytes, H.total)) return rc;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    float *x32 = reinterpret_cast<float *>(base + H.off_x), *y32 = reinterpret_cast<float *>(base + H.off_y);
    {
        ProfScope ps("widen_inputs", st);
        const int bf = input_type == SDTW_INPUT_BF16;
        widen_half_kernel<<<fill_grid((size_t)H.nx), 256, 0, st>>>(static_cast<const uint16_t *>(x), x32, (size_t)H.nx, bf);
        widen_half_kernel<<<fill_grid((size_t)H.ny), 256, 0, st>>>(static_cast<const uint16_t *>(y), y32, (size_t)H.ny, bf);
    }
    return forward_impl(desc, x32, y32, value, workspace, st, nullptr, nullptr, 1);
}

int sdtw_backward_half(const sdtw_desc *desc, const float *grad_value, float *dx, float *dy, float *E_out,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->flags & SDTW_FLAG_VALUE_ONLY) return SDTW_ERR_STATE;
    const HalfLayout H = half_layout(desc);
    if (int rc = check_ws(workspace, workspace_bytes, H.total)) return rc;
    char *base = static_cast<char *>(workspace);
    const float *x32 = reinterpret_cast<const float *>(base + H.off_x), *y32 = reinterpret_cast<const float *>(base + H.off_y);
    return backward_impl(desc, x32, y32, grad_value, dx, dy, E_out, workspace, static_cast<hipStream_t>(stream), nullptr,
                         nullptr, 1);
}

size_t sdtw_barycenter_workspace_bytes(const sdtw_bary_desc *desc)
{
    if (!bary_ok(desc)) return 0;
    return bary_layout(desc).total;
}

int sdtw_barycenter_step(const sdtw_bary_desc *desc, float *z, const float *X, float *adam_m, float *adam_v,
                         float *loss, float *dz_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!bary_ok(desc)) return SDTW_ERR_INVALID_ARG;
    if (!z || !X || !adam_m || !adam_v || !loss) return SDTW_ERR_INVALID_ARG;
    const BaryLayout BL = bary_layout(desc);
    if (int rc = check_ws(workspace, workspace_bytes, BL.total)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    float *values = reinterpret_cast<float *>(base + BL.off_values);
    float *dxk = reinterpret_cast<float *>(base + BL.off_dx);
    void *pair_ws = base + BL.off_pair_ws;
    const sdtw_desc s = bary_pair_desc(desc);
    if (int rc = forward_impl(&s, z, X, values, pair_ws, st)) return rc;
    if (int rc = backward_impl(&s, z, X, nullptr, dxk, nullptr, nullptr, pair_ws, st)) return rc;
    AdamParams a{};
    a.K = desc->K;
    a.n = (int64_t)desc->Lz * desc->D;
    a.lr = desc->lr; a.beta1 = desc->beta1; a.beta2 = desc->beta2; a.eps = desc->eps;
    a.corr1 = (float)(1.0 - std::pow((double)desc->beta1, (double)desc->step));
    a.corr2 = (float)(1.0 - std::pow((double)desc->beta2, (double)desc->step));
    {
        ProfScope ps("barycenter_update", st);
        barycenter_update_kernel<<<(unsigned)((a.n + 255) / 256), 256, 0, st>>>(
            a, reinterpret_cast<const Header *>(pair_ws), dxk, values, z, adam_m, adam_v, loss, dz_out);
    }
    return hip_ok();
}

size_t sdtw_normalized_workspace_bytes(const sdtw_desc *desc)
{
    int why;
    if (!desc_ok(desc, &why) || desc->bandwidth != 0) return 0;
    return norm_plan(desc).total;
}

int sdtw_normalized_forward(const sdtw_desc *desc, const float *x, const float *y, float *value, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->bandwidth != 0) return SDTW_ERR_UNSUPPORTED;
    if (!x || !y || !value) return SDTW_ERR_INVALID_ARG;
    const NormPlan P = norm_plan(desc);
    if (int rc = check_ws(workspace, workspace_bytes, P.total)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    float *vals = reinterpret_cast<float *>(base + P.off_vals);
    float *vxy = vals, *vxx = vals + desc->B, *vyy = vals + 2 * (size_t)desc->B;
    if (P.batched) {
        float *xs = reinterpret_cast<float *>(base + P.off_xs), *ys = reinterpret_cast<float *>(base + P.off_ys);
        const int64_t per = (int64_t)desc->N * desc->D;
        const int vec = per % 4 == 0 && desc->x_batch_stride % 4 == 0 && desc->y_batch_stride % 4 == 0 && aligned16(x) &&
                        aligned16(y);
        normalized_gather_kernel<<<fill_grid(3 * (size_t)desc->B * per / (vec ? 4 : 1)), 256, 0, st>>>(
            x, y, desc->x_batch_stride, desc->y_batch_stride, xs, ys, desc->B, per, vec);
        if (int rc = forward_impl(&P.all, xs, ys, vals, base + P.off_all, st)) return rc;
        normalized_value_kernel<<<(desc->B + 255) / 256, 256, 0, st>>>(value, vxy, vxx, vyy, desc->B, 0, 0);
        return hip_ok();
    }
    if (int rc = forward_impl(&P.xy, x, y, vxy, base + P.off_xy, st)) return rc;
    if (int rc = forward_impl(&P.xx, x, x, vxx, base + P.off_xx, st)) return rc;
    if (int rc = forward_impl(&P.yy, y, y, vyy, base + P.off_yy, st)) return rc;
    normalized_value_kernel<<<(desc->B + 255) / 256, 256, 0, st>>>(value, vxy, vxx, vyy, desc->B, P.x_shared, P.y_shared);
    merge_status_kernel<<<1, 64, 0, st>>>(reinterpret_cast<Header *>(base + P.off_xy),
                                          reinterpret_cast<const Header *>(base + P.off_xx),
                                          reinterpret_cast<const Header *>(base + P.off_yy));
    return hip_ok();
}

int sdtw_normalized_backward(const sdtw_desc *desc, const float *x, const float *y, const float *grad_value,
                             float *dx, float *dy, void *workspace, size_t workspace_bytes, void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (desc->bandwidth != 0) return SDTW_ERR_UNSUPPORTED;
    if (!x || !y) return SDTW_ERR_INVALID_ARG;
    if (desc->flags & SDTW_FLAG_VALUE_ONLY) return SDTW_ERR_STATE;
    const NormPlan P = norm_plan(desc);
    if (int rc = check_ws(workspace, workspace_bytes, P.total)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *base = static_cast<char *>(workspace);
    if (P.batched) {
        const float *xs = reinterpret_cast<const float *>(base + P.off_xs), *ys = reinterpret_cast<const float *>(base + P.off_ys);
        float *dxs = reinterpret_cast<float *>(base + P.off_dxs), *dys = reinterpret_cast<float *>(base + P.off_dys);
        // (the operands are the copies the forward call gathered: the caller must not have changed x, y since)
        if (int rc = backward_impl(&P.all, xs, ys, nullptr, dxs, dy ? dys : nullptr, nullptr, base + P.off_all, st)) return rc;
        const int64_t per = (int64_t)desc->N * desc->D;
        normalized_batched_grad_kernel<<<fill_grid((size_t)desc->B * per), 256, 0, st>>>(dx, dy, dxs, dys, grad_value,
                                                                                      desc->B, per);
        return hip_ok();
    }
    float *gx = reinterpret_cast<float *>(base + P.off_gx), *gy = reinterpret_cast<float *>(base + P.off_gy);
    if (int rc = backward_impl(&P.xy, x, y, grad_value, dx, dy, nullptr, base + P.off_xy, st)) return rc;
    if (dx) {
        if (int rc = backward_impl(&P.xx, x, x, nullptr, gx, nullptr, nullptr, base + P.off_xx, st)) return rc;
        const int64_t per = (int64_t)desc->N * desc->D;
        normalized_grad_kernel<<<fill_grid((size_t)desc->B * per), 256, 0, st>>>(dx, gx, grad_value, desc->B, per, P.x_shared);
    }
    if (dy) {
        if (int rc = backward_impl(&P.yy, y, y, nullptr, gy, nullptr, nullptr, base + P.off_yy, st)) return rc;
        const int64_t per = (int64_t)desc->M * desc->D;
        normalized_grad_kernel<<<fill_grid((size_t)desc->B * per), 256, 0, st>>>(dy, gy, grad_value, desc->B, per, P.y_shared);
    }
    merge_status_kernel<<<1, 64, 0, st>>>(reinterpret_cast<Header *>(base + P.off_xy),
                                          reinterpret_cast<const Header *>(base + P.off_xx),
                                          reinterpret_cast<const Header *>(base + P.off_yy));
    return hip_ok();
}

int sdtw_workspace_status(const void *workspace, size_t workspace_bytes, void *stream, int32_t *device_status)
{
    if (!device_status) return SDTW_ERR_INVALID_ARG;
    if (int rc = check_ws(workspace, workspace_bytes, sizeof(Header))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Header h;
    if (hipMemcpyAsync(&h, workspace, sizeof(Header), hipMemcpyDeviceToHost, st) != hipSuccess) return SDTW_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return SDTW_ERR_HIP;
    *device_status = (h.magic == kMagic) ? h.status : SDTW_ERR_STATE;
    return SDTW_OK;
}

int sdtw_debug_export(const sdtw_desc *desc, const void *workspace, size_t workspace_bytes, int what, void *out,
                      void *stream)
{
    int why;
    if (!desc_ok(desc, &why)) return why;
    if (!out) return SDTW_ERR_INVALID_ARG;
    const Layout L = layout_of(desc);
    if (int rc = check_ws(workspace, workspace_bytes, L.total)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Params p = make_params(desc, L, nullptr, nullptr, const_cast<void *>(workspace));
    const size_t n = (size_t)desc->B * desc->N * desc->M;
    switch (what) {
        case SDTW_EXPORT_COST:
            if (desc->mode != SDTW_UNFUSED) return SDTW_ERR_INVALID_ARG;
            if (hipMemcpyAsync(out, p.cost, n * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return SDTW_ERR_HIP;
            return SDTW_OK;
        case SDTW_EXPORT_R:
            if (L.recompute) return SDTW_ERR_UNSUPPORTED;  // the table is not stored in this regime
            export_R_kernel<<<fill_grid(n), 256, 0, st>>>(p, static_cast<double *>(out));
            return hip_ok();
        case SDTW_EXPORT_E:
            if (L.compact_E) return SDTW_ERR_UNSUPPORTED;  // no dense E in this workspace: ask sdtw_backward for E_out
            export_E_kernel<<<fill_grid(n), 256, 0, st>>>(p, static_cast<float *>(out));
            return hip_ok();
        default:
            return SDTW_ERR_INVALID_ARG;
    }
}

int sdtw_debug_lane_shift(int32_t *out, void *stream)
{
    if (!out) return SDTW_ERR_INVALID_ARG;
    lane_shift_probe_kernel<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(out);
    return hip_ok();
}

int sdtw_debug_set_spin_limit(uint32_t polls)
{
    g_spin_limit = polls;
    return SDTW_OK;
}

int sdtw_debug_force_workgroup_shape(int bands_per_workgroup)
{
    if (bands_per_workgroup != 0 && bands_per_workgroup != 1 && bands_per_workgroup != 2 && bands_per_workgroup != 4)
        return SDTW_ERR_INVALID_ARG;
    g_force_slots = bands_per_workgroup;
    return SDTW_OK;
}

int sdtw_debug_rate_probe(int probe, int variant, int waves_per_simd, int iters, void *scratch, size_t scratch_bytes,
                          float *ms, void *stream)
{
    if (!ms || iters < 1 || iters > (1 << 20)) return SDTW_ERR_INVALID_ARG;
    if (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) return SDTW_ERR_INVALID_ARG;
    if (int rc = check_ws(scratch, scratch_bytes, probe::kScratchBytes)) return rc;
    (void)hipGetLastError();
    hipStream_t st = static_cast<hipStream_t>(stream);
    double *d = static_cast<double *>(scratch);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return SDTW_ERR_HIP;
    }
    int rc = SDTW_OK;
    if (!probe::launch(probe, variant, waves_per_simd, 10, d, st)) {  // warm-up (instruction cache, clocks)
        rc = SDTW_ERR_INVALID_ARG;
    } else {
        (void)hipEventRecord(e0, st);
        probe::launch(probe, variant, waves_per_simd, iters, d, st);
        (void)hipEventRecord(e1, st);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = SDTW_ERR_HIP;
        if (rc == SDTW_OK) rc = hip_ok();
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

int sdtw_debug_set_pool_blocks(long long blocks)
{
    g_pool_blocks = blocks;
    return SDTW_OK;
}

int sdtw_debug_profile(int enable)
{
    for (ProfEntry &e : g_prof) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    g_prof.clear();
    g_profile = enable != 0;
    return SDTW_OK;
}

int sdtw_debug_profile_read(char *names, size_t names_bytes, float *ms, int max_entries, int *count)
{
    if (!names || !ms || !count || max_entries < 0) return SDTW_ERR_INVALID_ARG;
    std::string joined;
    int n = 0;
    for (ProfEntry &e : g_prof) {
        if (n >= max_entries) break;
        if (hipEventSynchronize(e.b) != hipSuccess) return SDTW_ERR_HIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, e.a, e.b) != hipSuccess) return SDTW_ERR_HIP;
        ms[n++] = t;
        joined += e.name;
        joined += ';';
    }
    if (joined.size() + 1 > names_bytes) return SDTW_ERR_INVALID_ARG;
    std::memcpy(names, joined.c_str(), joined.size() + 1);
    *count = n;
    for (ProfEntry &e : g_prof) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    g_prof.clear();
    return SDTW_OK;
}

}  // extern "C"
