"""The entry point that allocates nothing (sdtw_forward_static_scratch) against sdtw_forward.

Two calls in a row on the library's one scratch buffer, the second with a smaller problem, so that
whatever the first call left in the buffer is there when the second one starts.  Bar: the value's
(1e-4 relative); the kernels and launch shapes are the same, so the values are in fact identical.
"""
import numpy as np
import pytest

import paper_2602_17206_amd as pkg
from paper_2602_17206_amd import binding, workloads

pytestmark = pytest.mark.gpu

VALUE_RTOL = 1e-4


@pytest.mark.parametrize("mode", [pkg.UNFUSED, pkg.FUSED])
def test_static_scratch_forward_matches_forward_twice_in_a_row(mode):
    import torch

    for seed, (B, N, M, D, gamma) in enumerate([(8, 200, 180, 16, 0.5), (3, 70, 50, 16, 0.5)]):
        print("static scratch: mode %d B=%d N=%d M=%d D=%d" % (mode, B, N, M, D), flush=True)
        x, y = workloads.normal_pairs(900 + seed, B, N, M, D)
        xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
        want, _, _ = pkg.sdtw_forward(xd, yd, gamma, mode)
        desc = binding.make_desc(B, N, M, D, gamma, mode)
        got = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        rc = binding.sdtw_forward_static_scratch(desc, xd, yd, got)
        assert rc == 0, binding.sdtw_status_string(rc)
        torch.cuda.synchronize()
        w, g = want.cpu().numpy().astype(np.float64), got.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(g))
        assert np.all(np.abs(g - w) <= VALUE_RTOL * np.maximum(np.abs(w), 1.0)), (g, w)
        np.testing.assert_array_equal(g, w)


def test_static_scratch_refuses_what_does_not_fit():
    import torch

    # B = 32, N = M = 1024, D = 128 needs a few hundred MB of table: refused on the host, nothing enqueued
    desc = binding.make_desc(32, 1024, 1024, 128, 0.1, pkg.FUSED, flags=binding.FLAG_VALUE_ONLY)
    assert pkg.sdtw_workspace_bytes(desc) > binding.STATIC_SCRATCH_BYTES
    x = torch.zeros((32, 1024, 128), dtype=torch.float32, device="cuda")
    value = torch.zeros(32, dtype=torch.float32, device="cuda")
    assert binding.sdtw_forward_static_scratch(desc, x, x, value) == binding.STATUS_WORKSPACE
