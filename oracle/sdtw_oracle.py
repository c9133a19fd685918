"""ctypes front end of the float64 CPU oracle (``sdtw_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg.  The recurrences, the cost and the gradient formulas live in the C
file, where each function names the passage of the paper it writes out; this module marshals
arguments for them.  Two combinations of plain calls are written here, in numpy, because they
are nothing but that: :func:`normalized` (the difference of three plain values and of their
gradients) and :func:`ragged_batch` (one plain call per sliced pair).

``SDTW_ORACLE_SANITIZE=1`` in the environment builds and loads the oracle with
``-fsanitize=address,undefined`` instead (``libsdtw_oracle_san.so``); the process then needs the
sanitizer runtime preloaded, which ``tests/test_oracle_sanitized.py`` arranges for a child
process that re-runs the pins.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sdtw_oracle.c")
_SANITIZE = os.environ.get("SDTW_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libsdtw_oracle_san.so" if _SANITIZE else "libsdtw_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_fp = ctypes.POINTER(ctypes.c_float)


SANITIZE_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=undefined"]


def build(force=False, sanitize=None):
    """Compile the oracle with gcc (-O2, OpenMP across pairs; or, with ``sanitize``, -O1 with the
    address and undefined-behaviour sanitizers).  Returns the library path."""
    sanitize = _SANITIZE if sanitize is None else bool(sanitize)
    lib = os.path.join(_HERE, "libsdtw_oracle_san.so" if sanitize else "libsdtw_oracle.so")
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        flags = SANITIZE_FLAGS if sanitize else ["-O2"]
        subprocess.check_call(["gcc"] + flags + ["-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", lib, _SRC, "-lm"])
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.sdtw_oracle_batch.restype = ctypes.c_int
        lib.sdtw_oracle_batch.argtypes = [
            _fp, _fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_int64, ctypes.c_int64, _dp, ctypes.c_int, _dp, _dp, _dp, _dp, ctypes.c_int]
        lib.sdtw_oracle_batch_banded.restype = ctypes.c_int
        lib.sdtw_oracle_batch_banded.argtypes = [
            _fp, _fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, _dp, ctypes.c_int, _dp, _dp, _dp, _dp, ctypes.c_int]
        lib.sdtw_oracle_from_cost_banded.restype = ctypes.c_int
        lib.sdtw_oracle_from_cost_banded.argtypes = [
            _dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_int, _dp, _dp, _dp]
        lib.sdtw_oracle_pair_tables.restype = ctypes.c_int
        lib.sdtw_oracle_pair_tables.argtypes = [
            _fp, _fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            _dp, _dp, _dp, _dp, _dp, _dp]
        lib.sdtw_oracle_from_cost.restype = ctypes.c_int
        lib.sdtw_oracle_from_cost.argtypes = [
            _dp, ctypes.c_int, ctypes.c_int, ctypes.c_double, _dp, _dp, _dp]
        lib.sdtw_oracle_barycenter_step.restype = ctypes.c_int
        lib.sdtw_oracle_barycenter_step.argtypes = [
            _dp, _fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_int,
            _dp, _dp, _dp, _dp, ctypes.c_int]
        lib.sdtw_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_fp)


def _f64_out(shape):
    a = np.empty(shape, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def max_threads():
    return int(_load().sdtw_oracle_max_threads())


def _band(bandwidth):
    return -1 if bandwidth is None else int(bandwidth)


def batch(x, y, gamma, grad_value=None, backward=True, want_E=False, nthreads=0, bandwidth=None):
    """x [B,N,D] or [N,D] (shared by every pair), y [B,M,D] or [M,D].  ``bandwidth`` w: only cells
    with |i-j| <= w belong to the grid (Sakoe-Chiba band; None = no band).

    Returns a dict with ``value`` [B] and, when ``backward``, ``dx`` [B,N,D], ``dy`` [B,M,D]
    (and ``E`` [B,N,M] when ``want_E``), all float64.
    """
    lib = _load()
    x, xp = _f32(x)
    y, yp = _f32(y)
    if x.ndim == 2 and y.ndim == 2:
        x = x[None]
        y = y[None]
        xp = x.ctypes.data_as(_fp)
        yp = y.ctypes.data_as(_fp)
    B = y.shape[0] if y.ndim == 3 else x.shape[0]
    N, D = x.shape[-2], x.shape[-1]
    M = y.shape[-2]
    assert y.shape[-1] == D
    xs = N * D if x.ndim == 3 else 0
    ys = M * D if y.ndim == 3 else 0
    if x.ndim == 3:
        assert x.shape[0] == B
    if y.ndim == 3:
        assert y.shape[0] == B
    value, vp = _f64_out((B,))
    out = {"value": value}
    dxp = dyp = Ep = None
    if backward:
        out["dx"], dxp = _f64_out((B, N, D))
        out["dy"], dyp = _f64_out((B, M, D))
        if want_E:
            out["E"], Ep = _f64_out((B, N, M))
    gp = None
    if grad_value is not None:
        gv = np.ascontiguousarray(grad_value, dtype=np.float64)
        assert gv.shape == (B,)
        gp = gv.ctypes.data_as(_dp)
    rc = lib.sdtw_oracle_batch_banded(xp, yp, B, N, M, D, float(gamma), _band(bandwidth), xs, ys, gp,
                                      int(bool(backward)), vp, dxp, dyp, Ep, int(nthreads))
    if rc != 0:
        raise RuntimeError("sdtw_oracle_batch failed with code %d" % rc)
    return out


def ragged_batch(x, y, x_len, y_len, gamma, grad_value=None, want_E=False, bandwidth=None):
    """Pairs of individual lengths inside padded tensors x [B,N,D], y [B,M,D] (Sec. 5: the lengths of
    the two sequences of a pair may differ; here also from pair to pair): pair b is the plain
    problem on x[b, :x_len[b]], y[b, :y_len[b]], one call of :func:`batch` each; gradients and E
    are zero beyond a pair's lengths."""
    x = np.asarray(x)
    y = np.asarray(y)
    B, N, D = x.shape
    M = y.shape[1]
    out = {"value": np.zeros(B), "dx": np.zeros((B, N, D)), "dy": np.zeros((B, M, D))}
    if want_E:
        out["E"] = np.zeros((B, N, M))
    for b in range(B):
        n = N if x_len is None else int(x_len[b])
        m = M if y_len is None else int(y_len[b])
        gv = None if grad_value is None else np.asarray(grad_value, dtype=np.float64)[b:b + 1]
        o = batch(x[b:b + 1, :n], y[b:b + 1, :m], gamma, grad_value=gv, want_E=want_E, bandwidth=bandwidth)
        out["value"][b] = o["value"][0]
        out["dx"][b, :n] = o["dx"][0]
        out["dy"][b, :m] = o["dy"][0]
        if want_E:
            out["E"][b, :n, :m] = o["E"][0]
    return out


def normalized(x, y, gamma, grad_value=None, backward=True, nthreads=0):
    """Normalised Soft-DTW (Sec. 6, the normalisation paragraph):
    value = sdtw(x,y) - (sdtw(x,x) + sdtw(y,y)) / 2 per pair, written out as three plain calls
    of :func:`batch`; the self terms are differentiated with respect to both of their arguments.
    x [B,N,D], y [B,M,D] (N and M need not be equal here: each self term is a square problem of
    its own).  Returns ``value`` [B] and, when ``backward``, ``dx``, ``dy``; the three plain values
    are returned as ``parts`` [3,B] (xy, xx, yy)."""
    x = np.asarray(x)
    y = np.asarray(y)
    xy = batch(x, y, gamma, grad_value=grad_value, backward=backward, nthreads=nthreads)
    xx = batch(x, x, gamma, grad_value=grad_value, backward=backward, nthreads=nthreads)
    yy = batch(y, y, gamma, grad_value=grad_value, backward=backward, nthreads=nthreads)
    out = {"value": xy["value"] - 0.5 * (xx["value"] + yy["value"]),
           "parts": np.stack([xy["value"], xx["value"], yy["value"]])}
    if backward:
        out["dx"] = xy["dx"] - 0.5 * (xx["dx"] + xx["dy"])
        out["dy"] = xy["dy"] - 0.5 * (yy["dx"] + yy["dy"])
    return out


def pair_tables(x, y, gamma):
    """One pair x [N,D], y [M,D]; returns value, d [N,M], R [(N+2),(M+2)], E [N,M], dx, dy."""
    lib = _load()
    x, xp = _f32(x)
    y, yp = _f32(y)
    N, D = x.shape
    M = y.shape[0]
    assert y.shape[1] == D
    val = ctypes.c_double()
    d, dp_ = _f64_out((N, M))
    R, Rp = _f64_out((N + 2, M + 2))
    E, Ep = _f64_out((N, M))
    dx, dxp = _f64_out((N, D))
    dy, dyp = _f64_out((M, D))
    rc = lib.sdtw_oracle_pair_tables(xp, yp, N, M, D, float(gamma), ctypes.byref(val), dp_, Rp, Ep, dxp, dyp)
    if rc != 0:
        raise RuntimeError("sdtw_oracle_pair_tables failed with code %d" % rc)
    return {"value": val.value, "d": d, "R": R, "E": E, "dx": dx, "dy": dy}


def from_cost(d, gamma, want_E=True, bandwidth=None):
    """Forward (+ backward) on a given cost matrix d [N,M] (float64), optionally inside a band."""
    lib = _load()
    d = np.ascontiguousarray(d, dtype=np.float64)
    N, M = d.shape
    val = ctypes.c_double()
    R, Rp = _f64_out((N + 2, M + 2))
    E = Ep = None
    if want_E:
        E, Ep = _f64_out((N, M))
    rc = lib.sdtw_oracle_from_cost_banded(d.ctypes.data_as(_dp), N, M, float(gamma), _band(bandwidth),
                                          ctypes.byref(val), Rp, Ep)
    if rc != 0:
        raise RuntimeError("sdtw_oracle_from_cost failed with code %d" % rc)
    return {"value": val.value, "R": R, "E": E}


def barycenter_step(z, X, gamma, lr, beta1, beta2, eps, step, m, v, nthreads=0):
    """One Adam step on z (float64 arrays z, m, v are updated in place).  Returns (loss, dz)."""
    lib = _load()
    X, Xp = _f32(X)
    K, Lx, D = X.shape
    Lz = z.shape[0]
    for a in (z, m, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous and a.shape == (Lz, D)
    loss = ctypes.c_double()
    dz, dzp = _f64_out((Lz, D))
    rc = lib.sdtw_oracle_barycenter_step(
        z.ctypes.data_as(_dp), Xp, K, Lz, Lx, D, float(gamma), float(lr), float(beta1), float(beta2),
        float(eps), int(step), m.ctypes.data_as(_dp), v.ctypes.data_as(_dp), ctypes.byref(loss), dzp,
        int(nthreads))
    if rc != 0:
        raise RuntimeError("sdtw_oracle_barycenter_step failed with code %d" % rc)
    return loss.value, dz
