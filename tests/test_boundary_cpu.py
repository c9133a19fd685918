"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
symbol the header declares, sizes workspaces, and rejects bad arguments before any device work."""
import ctypes
import os
import re

import pytest

import paper_2602_17206_amd as pkg
from paper_2602_17206_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "sdtw.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdtw_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = pkg.load_library()
    names = header_functions()
    assert {"sdtw_forward", "sdtw_backward", "sdtw_barycenter_step", "sdtw_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    assert pkg.sdtw_version() >= 100
    assert pkg.sdtw_status_string(0) == "ok"
    assert "bandwidth" in pkg.sdtw_status_string(binding.STATUS_UNSUPPORTED)


def test_the_binding_loads_pytorch_before_the_library():
    # PyTorch's wheel carries a HIP runtime of its own; the library must bind to that one (the one the
    # tensors live in), which it does when it is loaded second.  A fresh interpreter that touches the
    # binding first must therefore find torch imported by the time the library is.
    import subprocess
    import sys

    code = ("import sys; import paper_2602_17206_amd as pkg; assert 'torch' not in sys.modules; "
            "pkg.sdtw_version(); assert 'torch' in sys.modules; print('ok')")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stderr[-2000:]


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(binding.Desc) == 48
    assert ctypes.sizeof(binding.BaryDesc) == 48


def test_workspace_sizes():
    # small problems (up to 1536 band tasks): float64 tables of both sweeps, float32 E
    d_f = binding.make_desc(32, 1024, 1024, 128, 0.1, pkg.FUSED)
    d_u = binding.make_desc(32, 1024, 1024, 128, 0.1, pkg.UNFUSED)
    wf, wu = pkg.sdtw_workspace_bytes(d_f), pkg.sdtw_workspace_bytes(d_u)
    cells = 32 * 1024 * 1024
    assert 4 * cells - 4096 <= wu - wf <= 4 * cells   # the cost tensor exists only in unfused mode
    split = 2 * 32 * 1024 * (128 * 2 * 2 + 4)         # float16 split copies of x, y and their scales
    assert 20 * cells < wf < 22 * cells + split       # 2 x (8 B + skew padding) + 4 B
    # value only: one table
    d_v = binding.make_desc(32, 1024, 1024, 128, 0.1, pkg.FUSED, flags=pkg.FLAG_VALUE_ONLY)
    wv = pkg.sdtw_workspace_bytes(d_v)
    assert 8 * cells < wf - wv < 9 * cells
    # large problems keep checkpoints instead of the tables and no E at all (fused: under a byte per cell)
    d_l = binding.make_desc(32, 8192, 8192, 128, 0.01, pkg.FUSED)
    assert pkg.sdtw_workspace_bytes(d_l) < 1.0 * 32 * 8192 * 8192
    d_lu = binding.make_desc(32, 8192, 8192, 128, 0.01, pkg.UNFUSED)
    assert 4.0 * 32 * 8192 * 8192 < pkg.sdtw_workspace_bytes(d_lu) < 5.0 * 32 * 8192 * 8192
    # ... and so do small ones on request
    d_m = binding.make_desc(32, 1024, 1024, 128, 0.1, pkg.FUSED, flags=pkg.FLAG_MIN_MEMORY)
    assert pkg.sdtw_workspace_bytes(d_m) < 2.5 * 32 * 1024 * 1024
    # long sequences with a dense E on request: 4 bytes per cell more
    d_d = binding.make_desc(32, 8192, 8192, 128, 0.01, pkg.FUSED, flags=pkg.FLAG_DENSE_E)
    assert 4.5 * 32 * 8192 * 8192 < pkg.sdtw_workspace_bytes(d_d) < 5.0 * 32 * 8192 * 8192
    # large problems of short pairs keep the dense E
    d_s = binding.make_desc(2048, 256, 256, 16, 1.0, pkg.FUSED)
    assert pkg.sdtw_workspace_bytes(d_s) > 4.0 * 2048 * 256 * 256
    assert pkg.sdtw_workspace_bytes(binding.make_desc(1, 1, 1, 1, 1.0, pkg.FUSED)) > 0
    # under a band constraint the tables follow the band, not M: E (4 B per cell of the full grid)
    # is what remains
    d_b = binding.make_desc(32, 8192, 8192, 64, 0.1, pkg.FUSED, bandwidth=128)
    cells = 32 * 8192 * 8192
    assert 4 * cells < pkg.sdtw_workspace_bytes(d_b) < 6 * cells
    d_bm = binding.make_desc(32, 8192, 8192, 64, 0.1, pkg.FUSED, bandwidth=128, flags=pkg.FLAG_MIN_MEMORY)
    assert pkg.sdtw_workspace_bytes(d_bm) < 0.6 * cells


@pytest.mark.parametrize("kw", [
    dict(B=0), dict(N=0), dict(M=-3), dict(D=0), dict(gamma=0.0), dict(gamma=-1.0), dict(gamma=float("nan")),
    dict(gamma=float("inf")), dict(mode=2), dict(mode=-1), dict(flags=8), dict(flags=6), dict(bandwidth=-1),
    dict(N=8, M=20, bandwidth=11),  # the last cell (N-1, M-1) would lie outside the band |i-j| <= 11
])
def test_invalid_descriptors_need_zero_bytes_and_are_refused(kw):
    args = dict(B=2, N=8, M=8, D=4, gamma=1.0, mode=pkg.FUSED)
    extra = {k: kw[k] for k in ("flags", "bandwidth") if k in kw}
    args.update({k: v for k, v in kw.items() if k not in extra})
    assert pkg.sdtw_workspace_bytes(binding.make_desc(2, 8, 20, 4, 1.0, pkg.FUSED, bandwidth=12)) > 0
    d = binding.make_desc(**args, **extra)
    assert pkg.sdtw_workspace_bytes(d) == 0
    lib = pkg.load_library()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: the descriptor is rejected first
    rc = lib.sdtw_forward(ctypes.byref(d), fake, fake, fake, fake, 1 << 30, None)
    assert rc == binding.STATUS_INVALID_ARG
    rc = lib.sdtw_backward(ctypes.byref(d), fake, fake, None, fake, fake, None, fake, 1 << 30, None)
    assert rc == binding.STATUS_INVALID_ARG


def test_normalized_entry_points_take_no_bandwidth():
    d = binding.make_desc(2, 8, 8, 4, 1.0, pkg.FUSED, bandwidth=3)
    assert pkg.sdtw_workspace_bytes(d) > 0
    assert pkg.sdtw_normalized_workspace_bytes(d) == 0
    lib = pkg.load_library()
    fake = ctypes.c_void_p(0x1000)  # never dereferenced
    assert lib.sdtw_normalized_forward(ctypes.byref(d), fake, fake, fake, fake, 1 << 30, None) == binding.STATUS_UNSUPPORTED
    assert lib.sdtw_normalized_backward(ctypes.byref(d), fake, fake, None, fake, fake, fake, 1 << 30, None) == binding.STATUS_UNSUPPORTED


def test_null_pointers_and_workspace_errors():
    lib = pkg.load_library()
    d = binding.make_desc(2, 8, 8, 4, 1.0, pkg.FUSED)
    need = pkg.sdtw_workspace_bytes(d)
    fake = ctypes.c_void_p(0x10000)
    assert lib.sdtw_forward(None, fake, fake, fake, fake, need, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_forward(ctypes.byref(d), None, fake, fake, fake, need, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_forward(ctypes.byref(d), fake, None, fake, fake, need, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_forward(ctypes.byref(d), fake, fake, None, fake, need, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_forward(ctypes.byref(d), fake, fake, fake, None, need, None) == binding.STATUS_WORKSPACE
    assert lib.sdtw_forward(ctypes.byref(d), fake, fake, fake, fake, need - 1, None) == binding.STATUS_WORKSPACE
    assert lib.sdtw_forward(ctypes.byref(d), fake, fake, fake, ctypes.c_void_p(0x10010), need, None) == binding.STATUS_WORKSPACE
    assert lib.sdtw_backward(ctypes.byref(d), None, fake, None, fake, fake, None, fake, need, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_backward(ctypes.byref(d), fake, fake, None, fake, fake, None, fake, need - 1, None) == binding.STATUS_WORKSPACE
    assert lib.sdtw_workspace_status(fake, need, None, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_debug_export(ctypes.byref(d), fake, need, 0, fake, None) == binding.STATUS_INVALID_ARG  # cost needs unfused
    assert lib.sdtw_debug_export(ctypes.byref(d), fake, need, 1, None, None) == binding.STATUS_INVALID_ARG
    assert lib.sdtw_debug_lane_shift(None, None) == binding.STATUS_INVALID_ARG


def test_barycenter_descriptor_checks():
    lib = pkg.load_library()
    good = binding.make_bary_desc(4, 16, 16, 2, 1.0, pkg.FUSED, 0.05, 0.9, 0.999, 1e-8, 1)
    need = pkg.sdtw_barycenter_workspace_bytes(good)
    assert need > 4 * 16 * 2 * 4
    fake = ctypes.c_void_p(0x10000)
    for field, bad in [("K", 0), ("Lz", 0), ("gamma", 0.0), ("lr", 0.0), ("beta1", 1.0), ("beta2", -0.1),
                       ("eps", 0.0), ("step", 0), ("mode", 7), ("flags", 1), ("flags", 4)]:
        d = binding.make_bary_desc(4, 16, 16, 2, 1.0, pkg.FUSED, 0.05, 0.9, 0.999, 1e-8, 1)
        setattr(d, field, bad)
        assert pkg.sdtw_barycenter_workspace_bytes(d) == 0, field
        assert lib.sdtw_barycenter_step(ctypes.byref(d), fake, fake, fake, fake, fake, None, fake, need, None) == \
            binding.STATUS_INVALID_ARG, field
    assert lib.sdtw_barycenter_step(ctypes.byref(good), None, fake, fake, fake, fake, None, fake, need, None) == \
        binding.STATUS_INVALID_ARG
    assert lib.sdtw_barycenter_step(ctypes.byref(good), fake, fake, fake, fake, fake, None, fake, need - 1, None) == \
        binding.STATUS_WORKSPACE


def test_workloads_are_seeded_and_shaped():
    import numpy as np
    from paper_2602_17206_amd import workloads as w

    a = w.pair_workload("c1_tiny")
    b = w.pair_workload("c1_tiny")
    assert a.x.shape == (4, 64, 8) and a.y.shape == (4, 64, 8) and a.x.dtype == np.float32 and a.gamma == 1.0
    np.testing.assert_array_equal(a.x, b.x)
    c = w.pair_workload("c3_b32_l1024_walk", B=2, N=64, M=48)
    assert c.x.shape == (2, 64, 128) and c.y.shape == (2, 48, 128)
    steps = np.diff(c.x.astype(np.float64), axis=1)
    assert 0.08 < steps.std() < 0.12                      # random-walk increments ~ N(0, 0.1)
    bw = w.barycenter_workload(K=6, L=40, D=3)
    assert bw.X.shape == (6, 40, 3) and bw.z0.shape == (40, 3)
    np.testing.assert_allclose(bw.z0, bw.X.mean(axis=0), rtol=1e-5, atol=1e-6)
