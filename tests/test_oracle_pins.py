"""Pins for the float64 CPU oracle (no GPU).  Each test fixes the oracle to something that
is not the oracle: enumeration of all alignment paths, closed forms, classic DTW, finite
differences, and invariants of the Soft-DTW definition (paper Sec. 2 and 4.2-4.4)."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def all_paths(N, M):
    """Every monotone path (1,1)->(N,M) with steps (1,0),(0,1),(1,1); 0-based cells."""
    out = []

    def rec(i, j, acc):
        acc = acc + [(i, j)]
        if i == N - 1 and j == M - 1:
            out.append(acc)
            return
        if i + 1 < N:
            rec(i + 1, j, acc)
        if j + 1 < M:
            rec(i, j + 1, acc)
        if i + 1 < N and j + 1 < M:
            rec(i + 1, j + 1, acc)

    rec(0, 0, [])
    return out


def brute_force(d, gamma):
    """value = -gamma log sum_paths exp(-cost/gamma); E[i,j] = P(path visits (i,j))."""
    N, M = d.shape
    paths = all_paths(N, M)
    costs = np.array([sum(d[i, j] for i, j in p) for p in paths])
    cmin = costs.min()
    w = np.exp(-(costs - cmin) / gamma)
    Z = w.sum()
    value = cmin - gamma * math.log(Z)
    E = np.zeros((N, M))
    for p, wp in zip(paths, w):
        for i, j in p:
            E[i, j] += wp / Z
    return value, E, len(paths)


def delannoy_table(n, m):
    T = np.zeros((n + 1, m + 1), dtype=object)
    for a in range(n + 1):
        for b in range(m + 1):
            T[a, b] = 1 if a == 0 or b == 0 else T[a - 1, b] + T[a, b - 1] + T[a - 1, b - 1]
    return T


def hard_dtw(d):
    N, M = d.shape
    R = np.full((N + 1, M + 1), np.inf)
    R[0, 0] = 0.0
    for i in range(1, N + 1):
        for j in range(1, M + 1):
            R[i, j] = d[i - 1, j - 1] + min(R[i - 1, j - 1], R[i - 1, j], R[i, j - 1])
    return R[N, M]


def grid_inputs(rng, shape, scale=1.0):
    """float32 values on a 2^-8 grid so that +-2^-10 perturbations are exact."""
    return (np.round(rng.standard_normal(shape) * scale * 256.0) / 256.0).astype(np.float32)


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("N,M", [(1, 1), (1, 5), (4, 1), (2, 2), (3, 5), (5, 3), (6, 6), (4, 7)])
@pytest.mark.parametrize("gamma", [1.0, 0.1, 0.01])
def test_value_and_E_match_path_enumeration(N, M, gamma):
    rng = np.random.default_rng(100 * N + M)
    d = rng.uniform(0.0, 2.0, size=(N, M))
    value, E, npaths = brute_force(d, gamma)
    o = oracle.from_cost(d, gamma)
    assert npaths == int(delannoy_table(N - 1, M - 1)[N - 1, M - 1])
    assert o["value"] == pytest.approx(value, rel=1e-12, abs=1e-12)
    np.testing.assert_allclose(o["E"], E, rtol=1e-9, atol=1e-12)


def test_every_R_entry_is_the_subproblem_value():
    rng = np.random.default_rng(7)
    d = rng.uniform(0.0, 3.0, size=(5, 6))
    gamma = 0.5
    R = oracle.from_cost(d, gamma)["R"]
    assert R[0, 0] == 0.0
    assert np.all(np.isinf(R[1:, 0])) and np.all(np.isinf(R[0, 1:]))
    for i in range(1, 6):
        for j in range(1, 7):
            v, _, _ = brute_force(d[:i, :j], gamma)
            assert R[i, j] == pytest.approx(v, rel=1e-12)


def test_pair_pipeline_matches_enumeration_through_x_and_y():
    rng = np.random.default_rng(11)
    N, M, D, gamma = 5, 4, 3, 0.3
    x = rng.standard_normal((N, D)).astype(np.float32)
    y = rng.standard_normal((M, D)).astype(np.float32)
    d = ((x[:, None, :].astype(np.float64) - y[None, :, :].astype(np.float64)) ** 2).sum(-1)
    value, E, _ = brute_force(d, gamma)
    o = oracle.pair_tables(x, y, gamma)
    np.testing.assert_allclose(o["d"], d, rtol=1e-14)
    assert o["value"] == pytest.approx(value, rel=1e-12)
    np.testing.assert_allclose(o["E"], E, rtol=1e-9, atol=1e-13)
    # gradient = sum over cells of E_ij * d(d_ij)/dx_i, d(d_ij)/dx_i = 2 (x_i - y_j)
    diff = x[:, None, :].astype(np.float64) - y[None, :, :].astype(np.float64)
    np.testing.assert_allclose(o["dx"], 2.0 * np.einsum("ij,ijk->ik", E, diff), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(o["dy"], -2.0 * np.einsum("ij,ijk->jk", E, diff), rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------- closed forms
def test_single_cell():
    x = np.array([[1.5, -2.0]], dtype=np.float32)
    y = np.array([[0.5, 1.0]], dtype=np.float32)
    o = oracle.pair_tables(x, y, 0.7)
    assert o["value"] == pytest.approx(1.0 + 9.0)
    assert o["E"][0, 0] == 1.0
    np.testing.assert_allclose(o["dx"], 2.0 * (x - y))
    np.testing.assert_allclose(o["dy"], -2.0 * (x - y))


def test_single_row_has_one_path():
    rng = np.random.default_rng(3)
    d = rng.uniform(0, 1, size=(1, 9))
    o = oracle.from_cost(d, 0.2)
    assert o["value"] == pytest.approx(d.sum(), rel=1e-13)
    np.testing.assert_allclose(o["E"], 1.0, rtol=1e-12)


def test_two_by_two_closed_form():
    d = np.array([[0.3, 1.1], [0.7, 0.2]])
    g = 0.4
    expect = d[0, 0] + d[1, 1] - g * math.log(1.0 + math.exp(-d[0, 1] / g) + math.exp(-d[1, 0] / g))
    o = oracle.from_cost(d, g)
    assert o["value"] == pytest.approx(expect, rel=1e-13)
    Z = 1.0 + math.exp(-d[0, 1] / g) + math.exp(-d[1, 0] / g)
    np.testing.assert_allclose(o["E"], [[1.0, math.exp(-d[0, 1] / g) / Z], [math.exp(-d[1, 0] / g) / Z, 1.0]],
                               rtol=1e-12)


def test_golden_delannoy_counts():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "delannoy.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 10
    for n, m, cnt in rows:
        n, m, cnt = int(n), int(m), int(cnt)
        for gamma in (1.0, 0.25):
            o = oracle.from_cost(np.zeros((n, m)), gamma, want_E=False)
            assert o["value"] == pytest.approx(-gamma * math.log(cnt), rel=1e-12, abs=1e-13)


@pytest.mark.parametrize("N,M,gamma", [(20, 17, 1.0), (33, 64, 0.1)])
def test_zero_cost_tables_are_delannoy(N, M, gamma):
    T = delannoy_table(N, M)
    x = np.full((N, 3), 0.25, dtype=np.float32)
    y = np.full((M, 3), 0.25, dtype=np.float32)
    o = oracle.pair_tables(x, y, gamma)
    total = T[N - 1, M - 1]
    for i in range(1, N + 1):
        for j in range(1, M + 1):
            assert o["R"][i, j] == pytest.approx(-gamma * math.log(T[i - 1, j - 1]), rel=1e-11, abs=1e-12)
            e = float(T[i - 1, j - 1] * T[N - i, M - j]) / float(total)
            assert o["E"][i - 1, j - 1] == pytest.approx(e, rel=1e-9)
    np.testing.assert_allclose(o["dx"], 0.0, atol=1e-12)


# ----------------------------------------------------------------------------- gamma -> 0
@pytest.mark.parametrize("gamma", [1.0, 0.1, 1e-2, 1e-4])
def test_sandwich_against_classic_dtw(gamma):
    rng = np.random.default_rng(5)
    N, M = 23, 31
    x = rng.standard_normal((N, 4)).astype(np.float32)
    y = rng.standard_normal((M, 4)).astype(np.float32)
    o = oracle.pair_tables(x, y, gamma)
    dtw = hard_dtw(o["d"])
    logdel = math.log(int(delannoy_table(N - 1, M - 1)[N - 1, M - 1]))
    assert o["value"] <= dtw + 1e-9
    assert o["value"] >= dtw - gamma * logdel - 1e-9
    if gamma <= 1e-4:
        assert o["value"] == pytest.approx(dtw, abs=gamma * logdel)
        # the alignment matrix collapses onto one path
        assert np.all((o["E"] < 1e-6) | (o["E"] > 1 - 1e-6))


# ----------------------------------------------------------------------------- finite differences
@pytest.mark.parametrize("gamma", [1.0, 0.1])
def test_gradients_match_central_differences(gamma):
    rng = np.random.default_rng(17)
    N, M, D = 7, 9, 3
    x = grid_inputs(rng, (N, D))
    y = grid_inputs(rng, (M, D))
    base = oracle.pair_tables(x, y, gamma)
    h = 2.0 ** -10

    def val(xx, yy):
        return oracle.batch(xx, yy, gamma, backward=False)["value"][0]

    for (i, k) in [(0, 0), (3, 1), (N - 1, 2), (2, 2)]:
        xp, xm = x.copy(), x.copy()
        xp[i, k] += h
        xm[i, k] -= h
        fd = (val(xp, y) - val(xm, y)) / (2 * h)
        assert base["dx"][i, k] == pytest.approx(fd, rel=2e-5, abs=1e-6)
    for (j, k) in [(0, 1), (4, 0), (M - 1, 2)]:
        yp, ym = y.copy(), y.copy()
        yp[j, k] += h
        ym[j, k] -= h
        fd = (val(x, yp) - val(x, ym)) / (2 * h)
        assert base["dy"][j, k] == pytest.approx(fd, rel=2e-5, abs=1e-6)


def test_E_is_the_derivative_with_respect_to_the_cost():
    rng = np.random.default_rng(19)
    d = rng.uniform(0.0, 2.0, size=(6, 8))
    g = 0.3
    E = oracle.from_cost(d, g)["E"]
    h = 1e-6
    for (i, j) in [(0, 0), (2, 3), (5, 7), (4, 1), (1, 6)]:
        dp, dm = d.copy(), d.copy()
        dp[i, j] += h
        dm[i, j] -= h
        fd = (oracle.from_cost(dp, g, False)["value"] - oracle.from_cost(dm, g, False)["value"]) / (2 * h)
        assert E[i, j] == pytest.approx(fd, rel=1e-6, abs=1e-9)


# ----------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("N,M,gamma", [(12, 12, 1.0), (9, 21, 0.1), (40, 25, 0.01)])
def test_invariants(N, M, gamma):
    rng = np.random.default_rng(N * 1000 + M)
    D = 5
    x = rng.standard_normal((N, D)).astype(np.float32)
    y = rng.standard_normal((M, D)).astype(np.float32)
    a = oracle.pair_tables(x, y, gamma)
    b = oracle.pair_tables(y, x, gamma)
    # symmetry of the definition
    assert a["value"] == pytest.approx(b["value"], rel=1e-13)
    np.testing.assert_allclose(a["E"], b["E"].T, rtol=1e-8, atol=1e-13)
    np.testing.assert_allclose(a["dx"], b["dy"], rtol=1e-8, atol=1e-11)
    E = a["E"]
    assert E.min() >= 0.0 and E.max() <= 1.0 + 1e-9
    assert E[0, 0] == pytest.approx(1.0, abs=1e-9) and E[-1, -1] == 1.0
    assert np.all(E.sum(axis=1) >= 1 - 1e-9) and np.all(E.sum(axis=0) >= 1 - 1e-9)
    assert max(N, M) - 1e-7 <= E.sum() <= N + M - 1 + 1e-7          # expected path length
    assert (E * a["d"]).sum() >= a["value"] - 1e-9                    # value = E[cost] - gamma*entropy
    # the cost depends on x - y only: a common shift changes nothing
    np.testing.assert_allclose(a["dx"].sum(axis=0) + a["dy"].sum(axis=0), 0.0, atol=1e-9 * max(1.0, np.abs(a["dx"]).max()))


def test_scaling_identity():
    rng = np.random.default_rng(23)
    x = rng.standard_normal((10, 4)).astype(np.float32)
    y = rng.standard_normal((13, 4)).astype(np.float32)
    s, g = 4.0, 0.8
    a = oracle.batch(s * x, s * y, g, backward=False)["value"][0]
    b = oracle.batch(x, y, g / (s * s), backward=False)["value"][0]
    assert a == pytest.approx(s * s * b, rel=1e-12)


def test_small_gamma_stays_finite_where_the_linear_form_overflows():
    # exp((R[i+1,j]-R[i,j]-d[i+1,j])/gamma) overflows for the weights below; the log-space
    # recurrence of Sec. 4.2 must still give finite E in [0,1].
    rng = np.random.default_rng(29)
    x = (10.0 * rng.standard_normal((48, 6))).astype(np.float32)
    y = (10.0 * rng.standard_normal((52, 6))).astype(np.float32)
    o = oracle.pair_tables(x, y, 1e-3)
    # rounding of R (ulp(R)/gamma per step, R ~ 1e4 here) is the only excess over 1
    assert np.all(np.isfinite(o["E"])) and o["E"].max() <= 1 + 1e-6
    assert np.all(np.isfinite(o["dx"])) and np.all(np.isfinite(o["dy"]))


# ----------------------------------------------------------------------------- batch plumbing
def test_batch_equals_pairs_and_broadcast_and_upstream_gradient():
    rng = np.random.default_rng(31)
    B, N, M, D, g = 3, 8, 11, 4, 0.5
    x = rng.standard_normal((B, N, D)).astype(np.float32)
    y = rng.standard_normal((B, M, D)).astype(np.float32)
    gv = np.array([1.0, -2.0, 0.5])
    o = oracle.batch(x, y, g, grad_value=gv, want_E=True)
    for b in range(B):
        p = oracle.pair_tables(x[b], y[b], g)
        assert o["value"][b] == p["value"]
        np.testing.assert_array_equal(o["E"][b], p["E"])
        np.testing.assert_allclose(o["dx"][b], gv[b] * p["dx"], rtol=1e-14)
        np.testing.assert_allclose(o["dy"][b], gv[b] * p["dy"], rtol=1e-14)
    ob = oracle.batch(x[0], y, g)           # one x shared by every pair
    for b in range(B):
        p = oracle.pair_tables(x[0], y[b], g)
        assert ob["value"][b] == p["value"]
        np.testing.assert_array_equal(ob["dx"][b], p["dx"])


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(37)
    x = rng.standard_normal((6, 20, 3)).astype(np.float32)
    y = rng.standard_normal((6, 17, 3)).astype(np.float32)
    a = oracle.batch(x, y, 0.2, nthreads=1)
    b = oracle.batch(x, y, 0.2, nthreads=4)
    for k in ("value", "dx", "dy"):
        np.testing.assert_array_equal(a[k], b[k])


# ----------------------------------------------------------------------------- barycenter step
# ----------------------------------------------------------------------------- normalised Soft-DTW
# ----------------------------------------------------------------------------- band |i-j| <= w
@pytest.mark.parametrize("N,M,w", [(5, 5, 1), (6, 6, 2), (4, 7, 3), (7, 5, 2), (6, 6, 0), (3, 6, 4)])
@pytest.mark.parametrize("gamma", [1.0, 0.05])
def test_band_matches_enumeration_of_the_paths_inside_it(N, M, w, gamma):
    # the banded problem is the sum over exactly those alignment paths all of whose cells satisfy
    # |i-j| <= w: enumerate them
    rng = np.random.default_rng(10 * N + M + w)
    d = rng.uniform(0.0, 2.0, size=(N, M))
    paths = [q for q in all_paths(N, M) if all(abs(i - j) <= w for i, j in q)]
    assert paths, "the corner must be inside the band"
    costs = np.array([sum(d[i, j] for i, j in q) for q in paths])
    wts = np.exp(-(costs - costs.min()) / gamma)
    value = costs.min() - gamma * math.log(wts.sum())
    E = np.zeros((N, M))
    for q, wq in zip(paths, wts):
        for i, j in q:
            E[i, j] += wq / wts.sum()
    o = oracle.from_cost(d, gamma, bandwidth=w)
    assert o["value"] == pytest.approx(value, rel=1e-12, abs=1e-12)
    np.testing.assert_allclose(o["E"], E, rtol=1e-9, atol=1e-12)
    ii, jj = np.indices((N, M))
    assert not o["E"][np.abs(ii - jj) > w].any()


def test_band_special_cases():
    rng = np.random.default_rng(5)
    N, M, D, gamma = 9, 11, 3, 0.4
    x = grid_inputs(rng, (N, D))
    y = grid_inputs(rng, (M, D))
    # a band that holds the whole grid changes nothing
    full = oracle.batch(x, y, gamma, want_E=True)
    wide = oracle.batch(x, y, gamma, want_E=True, bandwidth=max(N, M))
    for key in ("value", "dx", "dy", "E"):
        assert np.array_equal(full[key], wide[key])
    # w = 0 on a square problem leaves the diagonal path alone: value = sum_i d[i,i], E = identity
    d = rng.uniform(0.0, 2.0, size=(6, 6))
    o = oracle.from_cost(d, 0.3, bandwidth=0)
    assert o["value"] == pytest.approx(np.trace(d), rel=1e-14)
    np.testing.assert_allclose(o["E"], np.eye(6), rtol=0, atol=1e-14)
    # narrowing the band removes paths, so the value can only grow; and it is never below classic
    # DTW restricted to the band minus gamma log(#paths in the band)
    vals = [oracle.from_cost(d, 0.3, False, bandwidth=w)["value"] for w in (0, 1, 2, 3, 5)]
    assert all(a >= b - 1e-12 for a, b in zip(vals, vals[1:]))
    # the corner outside the band: no path, +inf
    assert oracle.from_cost(rng.uniform(size=(3, 7)), 0.3, False, bandwidth=2)["value"] == np.inf


def test_band_gradients_match_central_differences():
    rng = np.random.default_rng(23)
    N, M, D, gamma, w = 8, 10, 2, 0.5, 3
    x = grid_inputs(rng, (N, D))
    y = grid_inputs(rng, (M, D))
    base = oracle.batch(x, y, gamma, bandwidth=w)
    h = 2.0 ** -10

    def val(xx, yy):
        return oracle.batch(xx, yy, gamma, backward=False, bandwidth=w)["value"][0]

    for (i, k) in [(0, 0), (3, 1), (N - 1, 1)]:
        xp, xm = x.copy(), x.copy()
        xp[i, k] += h
        xm[i, k] -= h
        assert base["dx"][0, i, k] == pytest.approx((val(xp, y) - val(xm, y)) / (2 * h), rel=2e-5, abs=1e-6)
    for (j, k) in [(0, 1), (4, 0), (M - 1, 1)]:
        yp, ym = y.copy(), y.copy()
        yp[j, k] += h
        ym[j, k] -= h
        assert base["dy"][0, j, k] == pytest.approx((val(x, yp) - val(x, ym)) / (2 * h), rel=2e-5, abs=1e-6)


def test_ragged_batch_is_the_plain_problem_on_each_pair_s_own_prefix():
    # per pair against path enumeration on the sliced cost matrix; padding must not matter and the
    # gradients beyond the lengths are zero
    rng = np.random.default_rng(77)
    B, N, M, D, gamma = 3, 5, 4, 2, 0.6
    x = rng.standard_normal((B, N, D)).astype(np.float32).astype(np.float64)
    y = rng.standard_normal((B, M, D)).astype(np.float32).astype(np.float64)
    xl, yl = np.array([5, 2, 1]), np.array([3, 4, 1])
    out = oracle.ragged_batch(x, y, xl, yl, gamma, want_E=True)
    for b in range(B):
        n, m = xl[b], yl[b]
        d = ((x[b, :n, None, :] - y[b, None, :m, :]) ** 2).sum(-1)
        val, E, _ = brute_force(d, gamma)
        assert abs(out["value"][b] - val) < 1e-12
        assert np.abs(out["E"][b, :n, :m] - E).max() < 1e-12
        assert not out["E"][b, n:].any() and not out["E"][b, :, m:].any()
        assert not out["dx"][b, n:].any() and not out["dy"][b, m:].any()
        gx = 2 * (E[:, :, None] * (x[b, :n, None, :] - y[b, None, :m, :])).sum(1)
        assert np.abs(out["dx"][b, :n] - gx).max() < 1e-12
    x2, y2 = x.copy(), y.copy()
    x2[1, 2:] = 1e3
    y2[0, 3:] = -1e3
    out2 = oracle.ragged_batch(x2, y2, xl, yl, gamma)
    assert np.array_equal(out2["value"], out["value"]) and np.array_equal(out2["dy"], out["dy"])
    full = oracle.ragged_batch(x, y, None, None, gamma)
    assert np.array_equal(full["value"], oracle.batch(x, y, gamma)["value"])


def test_normalized_value_against_enumeration_and_classic_dtw():
    # Sec. 6 (normalisation): sdtw(x,y) - (sdtw(x,x) + sdtw(y,y))/2, each term pinned by path
    # enumeration on its own cost matrix; as gamma -> 0 the self terms vanish (DTW(x,x) = 0)
    rng = np.random.default_rng(23)
    x = grid_inputs(rng, (5, 2))
    y = grid_inputs(rng, (4, 2))

    def cost(a, b):
        return ((a[:, None, :].astype(np.float64) - b[None, :, :].astype(np.float64)) ** 2).sum(-1)

    for gamma in (1.0, 0.2):
        want = brute_force(cost(x, y), gamma)[0] - 0.5 * (brute_force(cost(x, x), gamma)[0] +
                                                           brute_force(cost(y, y), gamma)[0])
        got = oracle.normalized(x[None], y[None], gamma, backward=False)
        assert got["value"][0] == pytest.approx(want, rel=1e-12, abs=1e-12)
    g = 1e-5
    tiny = oracle.normalized(x[None], y[None], g, backward=False)
    logdel = math.log(int(delannoy_table(4, 4)[4, 4]))
    assert tiny["value"][0] == pytest.approx(hard_dtw(cost(x, y)), abs=2 * g * logdel)
    assert abs(tiny["parts"][1, 0]) <= g * logdel and abs(tiny["parts"][2, 0]) <= g * logdel


def test_normalized_is_zero_on_the_diagonal_symmetric_and_differentiable():
    rng = np.random.default_rng(29)
    B, N, M, D, gamma = 2, 8, 6, 3, 0.5
    x = grid_inputs(rng, (B, N, D))
    y = grid_inputs(rng, (B, M, D))
    same = oracle.normalized(x, x, gamma)
    np.testing.assert_allclose(same["value"], 0.0, atol=1e-12)
    np.testing.assert_allclose(same["dx"] + same["dy"], 0.0, atol=1e-12)  # a minimum along x = y
    a = oracle.normalized(x, y, gamma)
    b = oracle.normalized(y, x, gamma)
    np.testing.assert_allclose(a["value"], b["value"], rtol=1e-12)
    np.testing.assert_allclose(a["dx"], b["dy"], rtol=1e-10, atol=1e-12)
    assert np.all(a["value"] > 0)   # a divergence: positive for x != y on these inputs
    # finite differences through all three terms
    h = 2.0 ** -10

    def val(xx, yy):
        return oracle.normalized(xx, yy, gamma, backward=False)["value"]

    for (bb, i, k) in [(0, 0, 0), (1, 5, 2), (0, N - 1, 1)]:
        xp, xm = x.copy(), x.copy()
        xp[bb, i, k] += h
        xm[bb, i, k] -= h
        fd = (val(xp, y)[bb] - val(xm, y)[bb]) / (2 * h)
        assert a["dx"][bb, i, k] == pytest.approx(fd, rel=2e-5, abs=1e-6)
    for (bb, j, k) in [(1, 0, 1), (0, M - 1, 0)]:
        yp, ym = y.copy(), y.copy()
        yp[bb, j, k] += h
        ym[bb, j, k] -= h
        fd = (val(x, yp)[bb] - val(x, ym)[bb]) / (2 * h)
        assert a["dy"][bb, j, k] == pytest.approx(fd, rel=2e-5, abs=1e-6)
    # upstream gradient scales all three terms alike
    gv = np.array([2.0, -0.5])
    c = oracle.normalized(x, y, gamma, grad_value=gv)
    np.testing.assert_allclose(c["dx"], a["dx"] * gv[:, None, None], rtol=1e-12, atol=1e-14)


def test_barycenter_step_loss_gradient_and_first_adam_update():
    rng = np.random.default_rng(41)
    K, L, D, g = 5, 9, 2, 0.7
    X = rng.standard_normal((K, L, D)).astype(np.float32)
    z32 = rng.standard_normal((L, D)).astype(np.float32)
    z = z32.astype(np.float64)
    m = np.zeros((L, D))
    v = np.zeros((L, D))
    lr, b1, b2, eps = 0.05, 0.9, 0.999, 1e-8
    loss, dz = oracle.barycenter_step(z, X, g, lr, b1, b2, eps, 1, m, v)
    ref = oracle.batch(z32, X, g)
    assert loss == pytest.approx(ref["value"].sum(), rel=1e-14)
    np.testing.assert_allclose(dz, ref["dx"].sum(axis=0), rtol=1e-13)
    # first Adam step from zero moments: m_hat = dz, v_hat = dz^2  ->  step = lr*dz/(|dz|+eps)
    np.testing.assert_allclose(m, (1 - b1) * dz, rtol=1e-13)
    np.testing.assert_allclose(v, (1 - b2) * dz * dz, rtol=1e-13)
    np.testing.assert_allclose(z, z32 - lr * dz / (np.abs(dz) + eps), rtol=1e-12, atol=1e-15)
    # a second step uses the running moments
    z_before = z.copy()
    loss2, dz2 = oracle.barycenter_step(z, X, g, lr, b1, b2, eps, 2, m, v)
    m2 = b1 * (1 - b1) * dz + (1 - b1) * dz2
    v2 = b2 * (1 - b2) * dz * dz + (1 - b2) * dz2 * dz2
    np.testing.assert_allclose(m, m2, rtol=1e-12)
    np.testing.assert_allclose(z, z_before - lr * (m2 / (1 - b1 ** 2)) / (np.sqrt(v2 / (1 - b2 ** 2)) + eps),
                               rtol=1e-12, atol=1e-15)
    assert loss2 < loss
