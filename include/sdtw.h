/*
 * sdtw.h - C boundary of the MI355X (gfx950) Soft-DTW library.
 *
 * What is computed (paper: "SoftDTW-CUDA-Torch"):
 *   forward   R[i,j] = d(x_i,y_j) + softmin_gamma(R[i-1,j-1], R[i-1,j], R[i,j-1]),
 *             R[0,0]=0, R[i,0]=R[0,j]=+inf, value = R[N,M]              (Sec. 2, Eq. 1-3)
 *   cost      d(x_i,y_j) = ||x_i||^2 - 2<x_i,y_j> + ||y_j||^2            (Sec. 4.3, Eq. 8)
 *   backward  E[i,j] = dR[N,M]/dd[i,j] by the reverse DP carried in log space
 *             (Sec. 2 "Backward pass", Sec. 4.2), then
 *             dx_i = 2 (x_i sum_j E_ij - sum_j E_ij y_j), dy_j alike    (Sec. 4.3)
 *   modes     unfused: the B x N x M cost tensor is materialised once;
 *             fused:   the cost is recomputed per tile inside the DP kernels and the
 *                      cost tensor is never stored                       (Sec. 4.3)
 *   barycenter step: loss = sum_k sdtw(z, X_k), dz = sum_k d/dz, Adam    (Sec. 4.4)
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers to row-major, contiguous float32 memory
 *     owned by the caller, 16-byte aligned.  Descriptors and scalar out-parameters are
 *     HOST pointers.  Inputs are never modified; outputs are overwritten, not accumulated.
 *   - The library allocates no device memory.  Temporary storage is the caller's
 *     `workspace` (device, 256-byte aligned) of at least sdtw_workspace_bytes() bytes.  The
 *     forward call leaves its DP table there for the backward call of the same descriptor.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on it and return without waiting, except where stated.
 *   - Return value: an sdtw_status.  Argument errors are detected on the host before any
 *     device work is enqueued.  Conditions only the device can see (a backward call on a
 *     workspace whose forward was run for another descriptor; an inter-workgroup wait that
 *     gave up) are recorded in the workspace and read with sdtw_workspace_status().
 *   - No call throws, aborts or prints.
 *   - Two calls that use the same workspace must be ordered (same stream, or synchronised by
 *     the caller).
 */
#ifndef SDTW_H
#define SDTW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sdtw_status {
    SDTW_OK = 0,
    SDTW_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, gamma not finite or <= 0, bad mode,
                                 bandwidth < 0 or 0 < bandwidth < |N-M| */
    SDTW_ERR_WORKSPACE = 2,   /* workspace missing, misaligned or smaller than required */
    SDTW_ERR_UNSUPPORTED = 3, /* bandwidth != 0 in a normalised Soft-DTW call */
    SDTW_ERR_STATE = 4,       /* device: backward on a workspace not filled by a matching forward;
                                 host: backward with a SDTW_FLAG_VALUE_ONLY descriptor */
    SDTW_ERR_HIP = 5,         /* a HIP runtime call of this call failed (launch, copy); an error that an
                                 earlier, unrelated HIP call left pending is discarded at entry */
    SDTW_ERR_TIMEOUT = 6      /* device: a band gave up waiting for the band it depends on */
} sdtw_status;

enum { SDTW_UNFUSED = 0, SDTW_FUSED = 1 };

/*
 * sdtw_desc.flags.
 *   SDTW_FLAG_VALUE_ONLY: the caller wants sdtw_forward's value and will not call sdtw_backward
 *   with this descriptor (sdtw_backward returns SDTW_ERR_STATE).  Without it, for problems
 *   too small to fill the chip, sdtw_forward already runs the reverse sweep of the backward pass
 *   beside the forward sweep (it does not depend on the forward's table), so that sdtw_backward
 *   only has to combine the two tables.  The flag changes the workspace size.
 */
/*
 * How the alignment matrix E is kept between the reverse sweep and the gradient kernel.
 *   Problems too small to fill the chip keep both DP tables (16 bytes per cell) and a dense E.
 *   Large problems keep checkpoints of the forward sweep (0.5 bytes per cell) and
 *     - with fewer than 2^24 cells per pair (4096 x 4096): a dense float32 E [B,N,M] (4 bytes per cell);
 *     - with 2^24 cells per pair or more, D <= 128: a COMPACT E - only the 32x32 blocks that hold a
 *       non-zero, in a pool with room for 1/64 of all blocks (at least 2 (N/32 + M/32) per pair).  For
 *       the small gamma long alignments are run with, E is a few blocks wide around the alignment
 *       path and fits many times over.  If it does not fit, the backward call notices on the device
 *       and forms the gradients with a second reverse sweep that contracts every block of E into
 *       dx, dy while the block is on the chip: same result to rounding, several times slower.
 *   SDTW_FLAG_MIN_MEMORY: checkpoints and the compact E for any problem, however small or short
 *     (a fused workspace is then about 1 byte per cell or less).  Trades time for memory: small
 *     problems lose the two sweeps running side by side.
 *   SDTW_FLAG_DENSE_E: never the compact E: for long sequences whose E is known to be dense (large
 *     gamma), where the second sweep would cost more than the memory is worth.
 *   The two exclude each other.  Both change the workspace size; give the same flags to
 *   sdtw_workspace_bytes, the forward and the backward call.  SDTW_FLAG_MIN_MEMORY is also accepted in
 *   sdtw_bary_desc.flags.
 */
enum { SDTW_FLAG_VALUE_ONLY = 1, SDTW_FLAG_MIN_MEMORY = 2, SDTW_FLAG_DENSE_E = 4 };

/* What sdtw_debug_export copies out of a workspace. */
enum { SDTW_EXPORT_COST = 0, SDTW_EXPORT_R = 1, SDTW_EXPORT_E = 2 };

/* One batch of B independent pairs (x_b, y_b); every pair has the same N, M, D. */
typedef struct sdtw_desc {
    int32_t B, N, M, D;     /* all >= 1 */
    float gamma;            /* > 0, finite */
    int32_t mode;           /* SDTW_UNFUSED or SDTW_FUSED */
    int64_t x_batch_stride; /* elements between consecutive x sequences: N*D, or 0 = one x shared */
    int64_t y_batch_stride; /* elements between consecutive y sequences: M*D, or 0 = one y shared */
    int32_t bandwidth;      /* 0: no band constraint (as in the paper's Sec. 5).  w > 0: Algorithm 1's
                               `bandwidth`, read as the Sakoe-Chiba band: only cells with |i-j| <= w
                               (0-based i, j) belong to the grid; the others have cost +inf, E = 0.
                               Needs w >= |N-M| so that the last cell is inside; w >= max(N,M)
                               constrains nothing and is the same as 0.  With per-pair
                               lengths every pair needs |x_len[b]-y_len[b]| <= w, which the device
                               does not check: such a pair's value and gradients are undefined.  The
                               sweeps skip the macro-steps outside the band. */
    uint32_t flags;         /* 0 or an OR of SDTW_FLAG_VALUE_ONLY, SDTW_FLAG_MIN_MEMORY, SDTW_FLAG_DENSE_E */
} sdtw_desc;

/* One barycenter step: K sequences X_k [Lx,D] against the current barycenter z [Lz,D]. */
typedef struct sdtw_bary_desc {
    int32_t K, Lz, Lx, D;   /* all >= 1 */
    float gamma;            /* > 0, finite */
    int32_t mode;           /* SDTW_UNFUSED or SDTW_FUSED */
    float lr, beta1, beta2, eps; /* Adam: lr > 0, 0 <= beta < 1, eps > 0 */
    int32_t step;           /* 1-based index of this step (bias correction) */
    uint32_t flags;         /* 0 or SDTW_FLAG_MIN_MEMORY */
} sdtw_bary_desc;

int sdtw_version(void);
const char *sdtw_status_string(int status);

/* Bytes of workspace the descriptor needs; 0 if the descriptor is invalid.  Host only. */
size_t sdtw_workspace_bytes(const sdtw_desc *desc);

/*
 * Forward (Sec. 2 Eq. 1-3; Sec. 4.1 removes the length cap; Sec. 4.3 defines the modes).
 *   x [B,N,D] (or [N,D] with x_batch_stride 0), y [B,M,D]: device, read only.
 *   value [B]: device, out; value[b] = R[N,M] of pair b (float32; the table itself is
 *              carried in float64 inside the workspace).
 * Leaves the DP table (and, unfused, the cost tensor) in `workspace` for sdtw_backward.
 * For small problems (see SDTW_FLAG_VALUE_ONLY) the same launch also runs the reverse DP
 * T[i,j] = d[i,j] + softmin_gamma(T[i+1,j+1], T[i+1,j], T[i,j+1]), T[N+1,M+1] = 0, whose table the
 * backward call combines with R:  E[i,j] = exp((R[N,M] - R[i,j] - T[i,j] + d[i,j]) / gamma),
 * which is the log-space recurrence of Sec. 4.2 solved for E.
 */
int sdtw_forward(const sdtw_desc *desc, const float *x, const float *y, float *value,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * sdtw_forward for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops that only score pairs, harnesses that forbid hipMalloc.
 * Same arguments and result as sdtw_forward with SDTW_FLAG_VALUE_ONLY (the flag is implied: no
 * backward call can follow), but the workspace is a buffer of SDTW_STATIC_SCRATCH_BYTES that lives
 * inside the library's device image, one copy per GPU, held until the process ends.  The call
 * allocates nothing (no hipMalloc / hipFree, no events), enqueues the same kernels on `stream` and
 * returns without waiting.
 *   - A descriptor whose value-only workspace (sdtw_workspace_bytes with SDTW_FLAG_VALUE_ONLY set)
 *     exceeds SDTW_STATIC_SCRATCH_BYTES is refused with SDTW_ERR_WORKSPACE before anything is
 *     enqueued.
 *   - Every call on a GPU uses that GPU's one buffer and overwrites what the last call left there:
 *     calls that overlap on one GPU (different streams, or threads) race; order them.
 *   - The first call on a GPU looks the buffer's address up (hipGetSymbolAddress, no allocation):
 *     make that call outside graph capture.  The per-kernel timing hook (sdtw_debug_profile) must
 *     be off, since it creates events.
 *   - Device-side conditions cannot be read back (there is no workspace pointer to pass to
 *     sdtw_workspace_status); a band that gives up waiting leaves NaN-free but meaningless values,
 *     as for sdtw_forward.
 */
#define SDTW_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int sdtw_forward_static_scratch(const sdtw_desc *desc, const float *x, const float *y, float *value,
                                void *stream);

/*
 * Backward (Sec. 2 "Backward pass", Sec. 4.2 log-space recurrence, Sec. 4.3 gradient formulas).
 * Must follow sdtw_forward with the same descriptor, x, y and workspace.
 *   grad_value [B]: device, upstream dL/dvalue per pair, or NULL for ones.
 *   dx [B,N,D], dy [B,M,D]: device, out; either may be NULL if not wanted.  With
 *        x_batch_stride 0 dx still has one [N,D] slab per pair (the caller sums them).
 *   E_out [B,N,M]: device, out, optional (NULL): the alignment matrix E (entries that underflow
 *        float32 are exact zeros).  Where the workspace keeps E compactly (see the flags) the
 *        reverse sweep writes the non-zero blocks straight into E_out and the gradients are formed
 *        from there; without E_out nothing of size B x N x M exists anywhere (Sec. 4.3: the gradients
 *        "without ever materializing" such a tensor).  Both routes give the same dx, dy to rounding.
 */
int sdtw_backward(const sdtw_desc *desc, const float *x, const float *y, const float *grad_value,
                  float *dx, float *dy, float *E_out, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * Ragged batches: pair b uses only the first x_len[b] rows of x_b and the first y_len[b] rows of
 * y_b (Sec. 5 allows unequal lengths; here they may also differ from pair to pair).
 *   x_len, y_len [B]: device, int32, read only; either may be NULL (every pair has the full
 *        length N or M).  Values are clamped to [1, N] and [1, M].
 *   value[b] = sdtw(x_b[:x_len[b]], y_b[:y_len[b]]);  dx, dy and E are 0 beyond a pair's lengths.
 * Everything else as sdtw_forward / sdtw_backward (same descriptor and workspace size: the
 * tensors keep their padded shapes [B,N,D], [B,M,D]).  The backward call must be given the same
 * length vectors as the forward call (checked on the device by address: SDTW_ERR_STATE).
 */
int sdtw_forward_ragged(const sdtw_desc *desc, const float *x, const float *y, const int32_t *x_len,
                        const int32_t *y_len, float *value, void *workspace, size_t workspace_bytes,
                        void *stream);
int sdtw_backward_ragged(const sdtw_desc *desc, const float *x, const float *y, const int32_t *x_len,
                         const int32_t *y_len, const float *grad_value, float *dx, float *dy,
                         float *E_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Reduced-precision inputs (Sec. 6, "Mixed precision"): x and y given as float16 or bfloat16.
 *   x [B,N,D] (or [N,D] with x_batch_stride 0), y [B,M,D]: device, read only, 16-bit elements of the type
 *        `input_type` names; strides in the descriptor count elements, as always.
 *   value, grad_value, dx, dy, E_out: float32, as for sdtw_forward / sdtw_backward.
 * The forward call widens x and y to float32 copies inside the workspace (exact) and everything else
 * runs as for float32 inputs - tables in float64, exponentials in float32 - except the inner products of
 * the cost: a float16 / bfloat16 element is one float16 piece, not two, so the cost takes one matrix-core
 * product per 16 features instead of three.  The results are those of the rounded sequences to float32
 * accuracy (same bars as sdtw_forward against the oracle run on the rounded values).  What the rounding
 * itself does to the cost is the caller's to weigh against gamma: with relative rounding eps (2^-11 for
 * float16, 2^-8 for bfloat16), |d~ - d| <= 2 eps sqrt(d) sqrt(2 (||x_i||^2 + ||y_j||^2)), which has to stay
 * well below gamma for the alignment to be the one of the unrounded sequences.
 * The backward call reads the copies the forward call left in the workspace; it takes no x, y.
 * Workspace: sdtw_half_workspace_bytes (the plain workspace plus the two copies).  No per-pair lengths.
 */
enum { SDTW_INPUT_F16 = 1, SDTW_INPUT_BF16 = 2 };
size_t sdtw_half_workspace_bytes(const sdtw_desc *desc);
int sdtw_forward_half(const sdtw_desc *desc, const void *x, const void *y, int input_type, float *value,
                      void *workspace, size_t workspace_bytes, void *stream);
int sdtw_backward_half(const sdtw_desc *desc, const float *grad_value, float *dx, float *dy, float *E_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace for sdtw_barycenter_step; 0 if the descriptor is invalid.  Host only. */
size_t sdtw_barycenter_workspace_bytes(const sdtw_bary_desc *desc);

/*
 * One barycenter step (Sec. 4.4): loss = sum_k sdtw_gamma(z, X_k); dz = sum_k d sdtw/dz
 * (summed over k in index order); then Adam with bias correction:
 *   m = beta1 m + (1-beta1) dz;  v = beta2 v + (1-beta2) dz^2;
 *   z -= lr * (m/(1-beta1^step)) / (sqrt(v/(1-beta2^step)) + eps).
 *   z [Lz,D]: device, in/out.  X [K,Lx,D]: device, read only.
 *   adam_m, adam_v [Lz,D]: device, in/out, caller-owned optimiser state (zeros before step 1).
 *   loss [1]: device, out.  dz_out [Lz,D]: device, out, optional (NULL).
 * If the device reports an error for this step (sdtw_workspace_status: a band gave up waiting),
 * loss and dz_out are NaN and z, adam_m and adam_v are left unchanged.
 */
int sdtw_barycenter_step(const sdtw_bary_desc *desc, float *z, const float *X, float *adam_m,
                         float *adam_v, float *loss, float *dz_out, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Normalised Soft-DTW (Sec. 6, the normalisation paragraph):
 *   value[b] = sdtw(x_b, y_b) - (sdtw(x_b, x_b) + sdtw(y_b, y_b)) / 2,
 * three forward (and backward) passes through the kernels above: the cross term and the two self
 * terms, each self term a square problem of its own, so N and M need not be equal.  A sequence
 * shared by all pairs (batch stride 0) has its self term computed once.  The self terms are
 * symmetric in their two arguments, so d/dx of sdtw(x,x)/2 is the gradient with respect to the
 * first argument alone.  Arguments as for sdtw_forward / sdtw_backward (no E output); the
 * workspace holds the three plain workspaces and the self terms' gradients, and its status word
 * (sdtw_workspace_status) reports the worst of the three.
 * With N == M, no shared sequence and a batch small enough to leave the chip idle, the three terms
 * run as ONE batch of 3B pairs - (x_b,y_b), (x_b,x_b), (y_b,y_b) - on copies of x and y that the
 * forward call gathers into the workspace (which then holds one plain workspace of 3B pairs, the
 * copies and the batch's gradients): fewer, fuller launches.  The backward call uses those copies,
 * so, as for the plain calls, x and y must not change between the two.
 */
size_t sdtw_normalized_workspace_bytes(const sdtw_desc *desc);
int sdtw_normalized_forward(const sdtw_desc *desc, const float *x, const float *y, float *value,
                            void *workspace, size_t workspace_bytes, void *stream);
int sdtw_normalized_backward(const sdtw_desc *desc, const float *x, const float *y,
                             const float *grad_value, float *dx, float *dy, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * Reads the device-side status word of a workspace: waits for `stream`, copies 4 bytes to the
 * host.  *device_status receives SDTW_OK, SDTW_ERR_STATE or SDTW_ERR_TIMEOUT.  When a backward
 * call found SDTW_ERR_STATE its dx, dy and E outputs are filled with NaN.
 */
int sdtw_workspace_status(const void *workspace, size_t workspace_bytes, void *stream,
                          int32_t *device_status);

/*
 * Test hook: copies an intermediate out of a workspace as a plain row-major tensor.
 *   SDTW_EXPORT_COST: out = float32 [B,N,M], the cost tensor d (unfused mode, after forward)
 *   SDTW_EXPORT_R:    out = float64 [B,N,M], the DP table R[1..N,1..M] (after forward)
 *   SDTW_EXPORT_E:    out = float32 [B,N,M], the alignment matrix (after backward; SDTW_ERR_UNSUPPORTED
 *                     where the workspace keeps E compactly: use sdtw_backward's E_out there)
 * `out` is a device pointer with room for B*N*M elements of that type.
 */
int sdtw_debug_export(const sdtw_desc *desc, const void *workspace, size_t workspace_bytes,
                      int what, void *out, void *stream);

/*
 * Test hook: runs the two cross-lane shifts the DP kernels rely on, on lane numbers.
 * out [128] int32, device: out[t] = lane t-1 (lane 0: -1), out[64+t] = lane t+1 (lane 63: -2).
 */
int sdtw_debug_lane_shift(int32_t *out, void *stream);

/*
 * The sdtw_debug_set_spin_limit, sdtw_debug_force_workgroup_shape, sdtw_debug_set_pool_blocks and
 * sdtw_debug_profile hooks below
 * set process-wide switches (the only state this library keeps between calls).  They are for tests
 * and benchmarks: call them while no other thread is inside a call of this library, and do not
 * change the forced workgroup shape between sdtw_workspace_bytes, the forward and the backward call
 * of one problem (the shape decides the workspace layout).
 *
 * Test hook: number of polls after which a band that waits for its neighbouring band gives up
 * and records SDTW_ERR_TIMEOUT (default 2^23, several seconds).  Process-wide; host only.
 */
int sdtw_debug_set_spin_limit(uint32_t polls);

/*
 * Test hook: the DP kernels run one band per workgroup or two consecutive bands of a pair per
 * workgroup (problems of up to about 1536 band tasks), or four bands per workgroup (larger ones).
 * 1, 2 or 4 forces that shape for later calls whatever the size, 0 restores the choice by size.
 * Results agree across shapes to rounding.  The forced shape also decides the workspace layout, so
 * set it before sdtw_workspace_bytes.  Process-wide; host only.
 */
int sdtw_debug_force_workgroup_shape(int bands_per_workgroup);

/*
 * Test hook: capacity, in 32x32 blocks, of the pool of a compact E for later backward calls (never more
 * than the workspace was sized for; -1 restores that size).  A small value makes the pool run over,
 * which sends the backward call down its second, contracting sweep.  Process-wide; host only.
 */
int sdtw_debug_set_pool_blocks(long long blocks);

/*
 * Benchmark hook: per-kernel timing.  sdtw_debug_profile(1) makes every later call bracket each
 * of its kernel launches with two HIP events on the caller's stream (this creates events, so it
 * is not for latency-critical callers); sdtw_debug_profile(0) switches it off and drops what was
 * recorded.  sdtw_debug_profile_read waits for the recorded events, writes up to max_entries
 * durations in milliseconds to ms (host) and the kernel labels, ';'-separated in launch order, to
 * names (host, names_bytes long), sets *count and clears the record.  Process-wide; not
 * thread-safe.
 */
int sdtw_debug_profile(int enable);
int sdtw_debug_profile_read(char *names, size_t names_bytes, float *ms, int max_entries, int *count);

/*
 * Benchmark hook: calibration of the vector-ALU figures the DP sweeps are priced against.  Runs one
 * micro-kernel on 256 workgroups (one per compute unit), `iters` iterations of 32 instructions or
 * DP steps each after a short warm-up launch, waits, and writes the duration in milliseconds to
 * *ms (host).  Creates two HIP events per call.
 *   probe 0: issue rate of one instruction (variant 0..9: v_add_f32, v_fma_f32, v_add_f64, v_min_f64,
 *            v_fma_f64, v_exp_f32, v_log_f32, v_cvt_f32_f64, v_cvt_f64_f32, v_mov_b32_dpp), eight
 *            independent chains per wavefront, waves_per_simd (1, 2, 4) wavefronts per SIMD
 *   probe 1: the same instruction as one dependent chain (variants 0..6, 9), one wavefront per SIMD
 *   probe 2: the bare DP step of Sec. 2 Eq. 1-2 (one row per lane), waves_per_simd wavefronts per SIMD
 *   probe 3: the bare DP step with two rows per lane (128 cells per step and wavefront)
 *   probe 4: the DP step of one wavefront per SIMD beside a wavefront that issues `variant`
 *            v_mfma_f32_32x32x16_f16 per 32 steps (variant + 1000: two rows per lane)
 *   probe 5: the DP step of one wavefront per compute unit with the consumer's memory traffic;
 *            variant = bit set (1: cost from LDS, 2: edge value to LDS, 4: table store to HBM,
 *            8: a workgroup barrier per 32 steps); supported: 0, 1, 3, 7, 15, 4, 8
 *   scratch: device, 256-byte aligned, at least 16 MiB.
 */
int sdtw_debug_rate_probe(int probe, int variant, int waves_per_simd, int iters, void *scratch,
                          size_t scratch_bytes, float *ms, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SDTW_H */
