/*
 * Soft-DTW float64 CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU library is checked against.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product path never does.  It shares no code, header, table or
 * helper with the HIP sources.
 *
 * Everything is float64 and follows the paper's notation with 1-based (i,j):
 *   - cost           d[i,j] = sum_k (x[i,k]-y[j,k])^2       (Sec. 2: squared Euclidean,
 *                    written out directly, not through the norm expansion)
 *   - forward        R[i,j] = d[i,j] + softmin_g(R[i-1,j-1], R[i-1,j], R[i,j-1])
 *                    R[0,0]=0, R[i,0]=R[0,j]=+inf            (Sec. 2, Eq. 1-2)
 *   - value          sdtw = R[N,M]                           (Sec. 2, Eq. 3)
 *   - backward       Ebar[i,j] = logsumexp(Ebar[i+1,j]+alpha, Ebar[i,j+1]+beta,
 *                                          Ebar[i+1,j+1]+delta), Ebar[N,M]=0,
 *                    alpha=(R[i+1,j]-R[i,j]-d[i+1,j])/g and the same shape for the
 *                    other two successors; E=exp(Ebar)       (Sec. 4.2)
 *   - input grads    dx_i = 2 (x_i sum_j E_ij - sum_j E_ij y_j), dy_j likewise
 *                                                            (Sec. 4.3, last two equations)
 *   - barycenter     loss = sum_k sdtw(z, x^(k)), dz = sum_k d/dz, Adam update
 *                                                            (Sec. 4.4)
 *   - band           Algorithm 1 takes a `bandwidth` the paper does not define; the reading
 *                    here is the Sakoe-Chiba band: only cells with |i-j| <= w belong to the
 *                    grid.  The others are never visited: their R stays +inf, their Ebar
 *                    -inf (E = 0), exactly like the cells of the padding.  w < 0: no band.
 * Cells are visited in row-major order; there is no blocking, fusion or
 * reordering.  OpenMP is used only ACROSS pairs (each pair is independent).
 *
 * Out of memory: every function that allocates returns ORACLE_NO_MEM and leaves its outputs
 * unspecified; one_pair passes the code of the gradient step on, the batch returns the first one.
 *
 * Pins (tests/test_oracle_*.py, none needs a GPU): brute-force enumeration of all
 * monotone paths for N,M<=6 (value and E), the Delannoy closed form for zero
 * cost, the hard-DTW sandwich as gamma->0, central finite differences of the
 * value, symmetry / range / corner / translation / scaling invariants.
 * Parity unpinned: the barycenter *trajectory* over many steps (the paper fixes
 * neither Adam's constants nor the initial point); a single step's loss and
 * gradient are pinned through the functions above, and the Adam update is
 * pinned against a hand-evaluated closed form of its first step.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

/* softmin_g(a,b,c) = -g log(e^{-a/g}+e^{-b/g}+e^{-c/g})  (Sec. 2, Eq. 2), evaluated
 * with the minimum factored out.  At least one argument must be finite. */
static double softmin3(double a, double b, double c, double g)
{
    double m = a;
    if (b < m) m = b;
    if (c < m) m = c;
    double s = 0.0;
    if (a < INFINITY) s += exp(-(a - m) / g);
    if (b < INFINITY) s += exp(-(b - m) / g);
    if (c < INFINITY) s += exp(-(c - m) / g);
    return m - g * log(s);
}

/* logsumexp(a,b,c) = m + log(e^{a-m}+e^{b-m}+e^{c-m}), m = max  (Sec. 4.2).
 * Arguments equal to -inf contribute nothing; at least one must be finite. */
static double logsumexp3(double a, double b, double c)
{
    double m = a;
    if (b > m) m = b;
    if (c > m) m = c;
    double s = 0.0;
    if (a > -INFINITY) s += exp(a - m);
    if (b > -INFINITY) s += exp(b - m);
    if (c > -INFINITY) s += exp(c - m);
    return m + log(s);
}

/* d[(i-1)*M+(j-1)] = ||x_i - y_j||^2, i=1..N, j=1..M.  x is [N,D], y is [M,D]. */
void sdtw_oracle_cost(const float *x, const float *y, int N, int M, int D, double *d)
{
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < M; ++j) {
            double acc = 0.0;
            for (int k = 0; k < D; ++k) {
                double diff = (double)x[(size_t)i * D + k] - (double)y[(size_t)j * D + k];
                acc += diff * diff;
            }
            d[(size_t)i * M + j] = acc;
        }
}

/* Is cell (i,j) inside the band |i-j| <= w?  (w < 0: there is no band.) */
static int in_band(int i, int j, int w)
{
    if (w < 0) return 1;
    return (i > j ? i - j : j - i) <= w;
}

/* Forward table.  R has (N+2) x (M+2) entries (row stride M+2), indices 0..N+1 /
 * 0..M+1 as in Algorithm 1's padded table; row N+1 and column M+1 are left +inf
 * for the backward pass, and so is every cell outside the band.  Returns R[N,M]. */
double sdtw_oracle_forward_banded(const double *d, int N, int M, double gamma, int w, double *R)
{
    const size_t W = (size_t)M + 2;
    for (size_t q = 0; q < ((size_t)N + 2) * W; ++q) R[q] = INFINITY;
    R[0] = 0.0;
    for (int i = 1; i <= N; ++i)
        for (int j = 1; j <= M; ++j) {
            if (!in_band(i, j, w)) continue;
            const double a = R[(i - 1) * W + (j - 1)], b = R[(i - 1) * W + j], c = R[i * W + (j - 1)];
            if (!(a < INFINITY) && !(b < INFINITY) && !(c < INFINITY)) continue;  /* unreachable cell */
            R[i * W + j] = d[(size_t)(i - 1) * M + (j - 1)] + softmin3(a, b, c, gamma);
        }
    return R[(size_t)N * W + M];
}

double sdtw_oracle_forward(const double *d, int N, int M, double gamma, double *R)
{
    return sdtw_oracle_forward_banded(d, N, M, gamma, -1, R);
}

/* Log-space backward.  E is [N,M] (0-based storage of the 1-based matrix).  Ebar is
 * scratch of (N+2) x (M+2).  A successor outside 1..N x 1..M contributes -inf. */
void sdtw_oracle_backward_banded(const double *d, const double *R, int N, int M, double gamma, int w,
                                 double *Ebar, double *E)
{
    const size_t W = (size_t)M + 2;
    for (size_t q = 0; q < ((size_t)N + 2) * W; ++q) Ebar[q] = -INFINITY;
    Ebar[(size_t)N * W + M] = 0.0;
    for (int i = N; i >= 1; --i)
        for (int j = M; j >= 1; --j) {
            if (i == N && j == M) continue;
            if (!in_band(i, j, w)) continue;
            const double r = R[i * W + j];
            double ta = -INFINITY, tb = -INFINITY, tc = -INFINITY;
            if (i + 1 <= N && in_band(i + 1, j, w)) {
                double alpha = (R[(i + 1) * W + j] - r - d[(size_t)i * M + (j - 1)]) / gamma;
                ta = Ebar[(i + 1) * W + j] + alpha;
            }
            if (j + 1 <= M && in_band(i, j + 1, w)) {
                double beta = (R[i * W + (j + 1)] - r - d[(size_t)(i - 1) * M + j]) / gamma;
                tb = Ebar[i * W + (j + 1)] + beta;
            }
            if (i + 1 <= N && j + 1 <= M && in_band(i + 1, j + 1, w)) {
                double delta = (R[(i + 1) * W + (j + 1)] - r - d[(size_t)i * M + j]) / gamma;
                tc = Ebar[(i + 1) * W + (j + 1)] + delta;
            }
            if (ta > -INFINITY || tb > -INFINITY || tc > -INFINITY) Ebar[i * W + j] = logsumexp3(ta, tb, tc);
        }
    for (int i = 1; i <= N; ++i)
        for (int j = 1; j <= M; ++j)
            E[(size_t)(i - 1) * M + (j - 1)] = exp(Ebar[i * W + j]);
}

void sdtw_oracle_backward(const double *d, const double *R, int N, int M, double gamma,
                          double *Ebar, double *E)
{
    sdtw_oracle_backward_banded(d, R, N, M, gamma, -1, Ebar, E);
}

/* dx[i,:] = g * 2 (x_i sum_j E_ij - sum_j E_ij y_j); dy[j,:] = g * 2 (y_j sum_i E_ij - sum_i E_ij x_i).
 * Every sum runs over its index in increasing order; the feature loop is innermost only so that
 * memory is walked along rows (the terms of each sum and their order are those of the formula). */
int sdtw_oracle_input_grads(const float *x, const float *y, const double *E, int N, int M, int D,
                            double g, double *dx, double *dy)
{
    double *acc = (double *)malloc((size_t)(N > M ? N : M) * D * sizeof(double));
    double *marg = (double *)malloc((size_t)(N > M ? N : M) * sizeof(double));
    if (!acc || !marg) { free(acc); free(marg); return ORACLE_NO_MEM; }
    /* dx: for each i, sum over j */
    for (int i = 0; i < N; ++i) {
        double rs = 0.0;
        double *a = acc + (size_t)i * D;
        for (int k = 0; k < D; ++k) a[k] = 0.0;
        for (int j = 0; j < M; ++j) {
            const double e = E[(size_t)i * M + j];
            rs += e;
            for (int k = 0; k < D; ++k) a[k] += e * (double)y[(size_t)j * D + k];
        }
        for (int k = 0; k < D; ++k)
            dx[(size_t)i * D + k] = g * 2.0 * ((double)x[(size_t)i * D + k] * rs - a[k]);
    }
    /* dy: for each j, sum over i (i is the outer loop, so each j still receives its terms in order of i) */
    for (int j = 0; j < M; ++j) {
        marg[j] = 0.0;
        for (int k = 0; k < D; ++k) acc[(size_t)j * D + k] = 0.0;
    }
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < M; ++j) {
            const double e = E[(size_t)i * M + j];
            double *a = acc + (size_t)j * D;
            marg[j] += e;
            for (int k = 0; k < D; ++k) a[k] += e * (double)x[(size_t)i * D + k];
        }
    for (int j = 0; j < M; ++j)
        for (int k = 0; k < D; ++k)
            dy[(size_t)j * D + k] = g * 2.0 * ((double)y[(size_t)j * D + k] * marg[j] - acc[(size_t)j * D + k]);
    free(acc);
    free(marg);
    return ORACLE_OK;
}

/* One pair, start to end.  Any of R_out ((N+2)(M+2)), E_out (N*M), dx, dy, d_out (N*M)
 * may be NULL.  want_backward=0 stops after the value. */
static int one_pair(const float *x, const float *y, int N, int M, int D, double gamma, int w, double g,
                    int want_backward, double *value, double *dx, double *dy, double *E_out,
                    double *R_out, double *d_out)
{
    const size_t nm = (size_t)N * M, pad = ((size_t)N + 2) * ((size_t)M + 2);
    double *d = (double *)malloc(nm * sizeof(double));
    double *R = (double *)malloc(pad * sizeof(double));
    if (!d || !R) { free(d); free(R); return ORACLE_NO_MEM; }
    sdtw_oracle_cost(x, y, N, M, D, d);
    *value = sdtw_oracle_forward_banded(d, N, M, gamma, w, R);
    if (d_out) memcpy(d_out, d, nm * sizeof(double));
    if (R_out) memcpy(R_out, R, pad * sizeof(double));
    if (want_backward) {
        double *Ebar = (double *)malloc(pad * sizeof(double));
        double *E = E_out ? E_out : (double *)malloc(nm * sizeof(double));
        if (!Ebar || !E) { free(d); free(R); free(Ebar); if (!E_out) free(E); return ORACLE_NO_MEM; }
        sdtw_oracle_backward_banded(d, R, N, M, gamma, w, Ebar, E);
        int rc = ORACLE_OK;
        if (dx || dy) {
            double *tx = dx ? dx : (double *)malloc((size_t)N * D * sizeof(double));
            double *ty = dy ? dy : (double *)malloc((size_t)M * D * sizeof(double));
            rc = (tx && ty) ? sdtw_oracle_input_grads(x, y, E, N, M, D, g, tx, ty) : ORACLE_NO_MEM;
            if (!dx) free(tx);
            if (!dy) free(ty);
        }
        free(Ebar);
        if (!E_out) free(E);
        if (rc != ORACLE_OK) { free(d); free(R); return rc; }
    }
    free(d);
    free(R);
    return ORACLE_OK;
}

/* Batch of B independent pairs.  x: B sequences spaced x_stride elements apart (0 = every
 * pair uses the same x), y likewise.  grad_value (B) may be NULL (= ones).  Outputs:
 * value[B]; dx[B,N,D], dy[B,M,D], E[B,N,M] each optional (NULL).  nthreads<=0: OpenMP default.
 * Returns 0, or the first non-zero per-pair code. */
int sdtw_oracle_batch_banded(const float *x, const float *y, int B, int N, int M, int D, double gamma,
                             int w, int64_t x_stride, int64_t y_stride, const double *grad_value,
                             int want_backward, double *value, double *dx, double *dy, double *E,
                             int nthreads)
{
    if (!x || !y || !value || B < 1 || N < 1 || M < 1 || D < 1 || !(gamma > 0.0) || !isfinite(gamma))
        return ORACLE_BAD_ARG;
    int rc = ORACLE_OK;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int r = one_pair(x + (size_t)b * x_stride, y + (size_t)b * y_stride, N, M, D, gamma, w,
                         grad_value ? grad_value[b] : 1.0, want_backward, &value[b],
                         dx ? dx + (size_t)b * N * D : NULL, dy ? dy + (size_t)b * M * D : NULL,
                         E ? E + (size_t)b * N * M : NULL, NULL, NULL);
        if (r != ORACLE_OK) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

int sdtw_oracle_batch(const float *x, const float *y, int B, int N, int M, int D, double gamma,
                      int64_t x_stride, int64_t y_stride, const double *grad_value,
                      int want_backward, double *value, double *dx, double *dy, double *E,
                      int nthreads)
{
    return sdtw_oracle_batch_banded(x, y, B, N, M, D, gamma, -1, x_stride, y_stride, grad_value,
                                    want_backward, value, dx, dy, E, nthreads);
}

/* One pair with every intermediate exposed (for the pins). */
int sdtw_oracle_pair_tables(const float *x, const float *y, int N, int M, int D, double gamma,
                            double *value, double *d_out, double *R_out, double *E_out,
                            double *dx, double *dy)
{
    if (!x || !y || !value || N < 1 || M < 1 || D < 1 || !(gamma > 0.0) || !isfinite(gamma))
        return ORACLE_BAD_ARG;
    return one_pair(x, y, N, M, D, gamma, -1, 1.0, 1, value, dx, dy, E_out, R_out, d_out);
}

/* Forward and backward on a caller-supplied cost matrix d[N,M] (for pins that fix d). */
int sdtw_oracle_from_cost_banded(const double *d, int N, int M, double gamma, int w, double *value,
                                 double *R_out, double *E_out)
{
    if (!d || !value || N < 1 || M < 1 || !(gamma > 0.0) || !isfinite(gamma)) return ORACLE_BAD_ARG;
    const size_t pad = ((size_t)N + 2) * ((size_t)M + 2);
    double *R = (double *)malloc(pad * sizeof(double));
    double *Ebar = (double *)malloc(pad * sizeof(double));
    if (!R || !Ebar) { free(R); free(Ebar); return ORACLE_NO_MEM; }
    *value = sdtw_oracle_forward_banded(d, N, M, gamma, w, R);
    if (R_out) memcpy(R_out, R, pad * sizeof(double));
    if (E_out) sdtw_oracle_backward_banded(d, R, N, M, gamma, w, Ebar, E_out);
    free(R);
    free(Ebar);
    return ORACLE_OK;
}

int sdtw_oracle_from_cost(const double *d, int N, int M, double gamma, double *value,
                          double *R_out, double *E_out)
{
    return sdtw_oracle_from_cost_banded(d, N, M, gamma, -1, value, R_out, E_out);
}

/* Barycenter step (Sec. 4.4): loss = sum_k sdtw_g(z, X_k), dz = sum_k d sdtw/dz, then one
 * Adam update of z (Kingma & Ba, bias-corrected; step counts from 1):
 *   m = b1 m + (1-b1) dz;  v = b2 v + (1-b2) dz^2;
 *   z -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps).
 * z [Lz,D] (float64 in/out), X [K,Lx,D] float32, m,v [Lz,D] in/out, dz_out optional.
 * z is rounded to float32 before it enters the distance, since the library keeps z in float32. */
int sdtw_oracle_barycenter_step(double *z, const float *X, int K, int Lz, int Lx, int D, double gamma,
                                double lr, double beta1, double beta2, double eps, int step,
                                double *m, double *v, double *loss, double *dz_out, int nthreads)
{
    if (!z || !X || !m || !v || !loss || K < 1 || Lz < 1 || Lx < 1 || D < 1 || step < 1 ||
        !(gamma > 0.0) || !isfinite(gamma))
        return ORACLE_BAD_ARG;
    const size_t zn = (size_t)Lz * D;
    float *zf = (float *)malloc(zn * sizeof(float));
    double *val = (double *)malloc((size_t)K * sizeof(double));
    double *dxs = (double *)malloc((size_t)K * zn * sizeof(double));
    if (!zf || !val || !dxs) { free(zf); free(val); free(dxs); return ORACLE_NO_MEM; }
    for (size_t q = 0; q < zn; ++q) zf[q] = (float)z[q];
    int rc = sdtw_oracle_batch(zf, X, K, Lz, Lx, D, gamma, 0, (int64_t)Lx * D, NULL, 1, val, dxs, NULL,
                               NULL, nthreads);
    if (rc == ORACLE_OK) {
        double L = 0.0;
        for (int k = 0; k < K; ++k) L += val[k];
        *loss = L;
        const double c1 = 1.0 - pow(beta1, (double)step), c2 = 1.0 - pow(beta2, (double)step);
        for (size_t q = 0; q < zn; ++q) {
            double gsum = 0.0;
            for (int k = 0; k < K; ++k) gsum += dxs[(size_t)k * zn + q];
            if (dz_out) dz_out[q] = gsum;
            m[q] = beta1 * m[q] + (1.0 - beta1) * gsum;
            v[q] = beta2 * v[q] + (1.0 - beta2) * gsum * gsum;
            z[q] -= lr * (m[q] / c1) / (sqrt(v[q] / c2) + eps);
        }
    }
    free(zf);
    free(val);
    free(dxs);
    return rc;
}

int sdtw_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
