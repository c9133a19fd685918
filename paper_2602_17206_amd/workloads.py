"""Seeded synthetic inputs for the five benchmark configurations.

Only random-number recipes live here; none of Soft-DTW's arithmetic does.  The same arrays
are handed to the HIP library and to the CPU oracle.  The paper's own benchmark inputs are
unspecified random tensors of a given shape (Sec. 5), so these stand in for them; no public
dataset is involved.
"""
from collections import namedtuple

import numpy as np

PairWorkload = namedtuple("PairWorkload", "name B N M D gamma modes x y")
BarycenterWorkload = namedtuple("BarycenterWorkload", "name K L D gamma steps lr X z0 template")

CONFIG_SHAPES = {
    # name: (B, N, M, D, gamma, modes, kind, seed)
    "c1_tiny": (4, 64, 64, 8, 1.0, ("unfused",), "normal", 1),
    "c2_b32_l256": (32, 256, 256, 128, 0.1, ("unfused", "fused"), "normal", 2),
    "c3_b32_l1024_walk": (32, 1024, 1024, 128, 0.1, ("unfused", "fused"), "walk", 3),
    "c4_b32_l8192": (32, 8192, 8192, 128, 0.01, ("fused",), "normal", 4),
}


def normal_pairs(seed, B, N, M, D):
    """x [B,N,D], y [B,M,D] ~ N(0,1), float32."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, N, D), dtype=np.float32)
    y = rng.standard_normal((B, M, D), dtype=np.float32)
    return x, y


def walk_pairs(seed, B, N, M, D, step_std=0.1):
    """Smooth random walks: cumulative sum over time of N(0, step_std) steps, per feature."""
    rng = np.random.default_rng(seed)
    x = np.cumsum(step_std * rng.standard_normal((B, N, D)), axis=1).astype(np.float32)
    y = np.cumsum(step_std * rng.standard_normal((B, M, D)), axis=1).astype(np.float32)
    return x, y


def ragged_lengths(seed, B, full, shortest=1):
    """Per-pair lengths for a padded batch: uniform integers in [shortest, full], int32; pair 0 keeps
    the full length and pair B-1 (if B > 1) the shortest, so both ends are always present."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(shortest, full + 1, size=B).astype(np.int32)
    lens[0] = full
    if B > 1:
        lens[-1] = shortest
    return lens


def pair_workload(name, B=None, N=None, M=None, D=None):
    """One of CONFIG_SHAPES by name; B/N/M/D override the shape (same recipe and seed)."""
    b, n, m, d, gamma, modes, kind, seed = CONFIG_SHAPES[name]
    B, N, M, D = B or b, N or n, M or m, D or d
    x, y = (normal_pairs if kind == "normal" else walk_pairs)(seed, B, N, M, D)
    return PairWorkload(name, B, N, M, D, gamma, modes, x, y)


def barycenter_workload(K=64, L=512, D=32, seed=5, gamma=1.0, steps=50, lr=0.05, noise=0.05):
    """K noisy, monotonically time-warped copies of a sine-mixture template.

    template[n,f] = sum_{h<3} a_hf sin(2 pi w_hf u_n + phi_hf), u_n = n/(L-1), a~U(0.5,1),
    w in {1..5}, phi~U(0,2pi).  Copy k samples the template at warped times tau_k (normalised
    cumulative sum of Gamma(4,1) increments, tau_k[0]=0, tau_k[L-1]=1) and adds
    noise*N(0,1).  z0 is the element-wise mean of the copies.
    """
    rng = np.random.default_rng(seed)
    a = rng.uniform(0.5, 1.0, size=(3, D))
    w = rng.integers(1, 6, size=(3, D)).astype(np.float64)
    phi = rng.uniform(0.0, 2.0 * np.pi, size=(3, D))

    def tmpl(u):  # u [...], returns [..., D]
        return np.sum(a * np.sin(2.0 * np.pi * w * u[..., None, None] + phi), axis=-2)

    u = np.linspace(0.0, 1.0, L)
    template = tmpl(u)
    inc = rng.gamma(4.0, 1.0, size=(K, L - 1))
    tau = np.concatenate([np.zeros((K, 1)), np.cumsum(inc, axis=1)], axis=1)
    tau /= tau[:, -1:]
    X = tmpl(tau) + noise * rng.standard_normal((K, L, D))
    X = X.astype(np.float32)
    z0 = X.astype(np.float64).mean(axis=0).astype(np.float32)
    return BarycenterWorkload("c5_barycenter", K, L, D, gamma, steps, lr, X, z0, template.astype(np.float32))
