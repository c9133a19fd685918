"""Parity of the HIP path against the float64 CPU oracle, element by element, through the C-ABI.

Bars (stated by the benchmark spec for fp32 I/O): |value - oracle| <= 1e-4 * max(|oracle|, 1) per pair;
max|dx - oracle| <= 1e-3 * max|oracle dx| per pair (dy alike).  E is compared with an absolute
tolerance since its entries lie in [0, 1].
"""
import sys

import numpy as np
import pytest

import oracle
import paper_2602_17206_amd as pkg
from paper_2602_17206_amd import binding, workloads

pytestmark = pytest.mark.gpu

VALUE_RTOL = 1e-4
GRAD_RTOL = 1e-3
E_ATOL = 2e-4
MODES = {"unfused": pkg.UNFUSED, "fused": pkg.FUSED}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_gpu(x, y, gamma, mode, grad_value=None, want_E=True, min_memory=False):
    import torch

    xd, yd = to_dev(x), to_dev(y)
    value, desc, ws = pkg.sdtw_forward(xd, yd, gamma, mode, min_memory=min_memory)
    gv = to_dev(grad_value.astype(np.float32)) if grad_value is not None else None
    # The gradients come from the call without E output: where the workspace keeps no E (large problems,
    # SDTW_FLAG_MIN_MEMORY) that is the reverse sweep that contracts E block by block.  E comes from a
    # second backward call on the same workspace, whose gradients (formed from the stored E there) must agree.
    dx, dy, _ = pkg.sdtw_backward(desc, xd, yd, ws, grad_value=gv)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    out = {"value": value.cpu().numpy().astype(np.float64), "dx": dx.cpu().numpy().astype(np.float64),
           "dy": dy.cpu().numpy().astype(np.float64), "desc": desc, "ws": ws}
    if want_E:
        dx2, dy2, E = pkg.sdtw_backward(desc, xd, yd, ws, grad_value=gv, want_E=True)
        torch.cuda.synchronize()
        assert binding.workspace_status(ws) == 0
        out["E"] = E.cpu().numpy().astype(np.float64)
        assert_same_gradients(dx, dx2, dy, dy2, xd, yd)
    return out


def assert_same_gradients(dx, dx2, dy, dy2, xd, yd):
    """Two routes to the same gradients agree to rounding.  Each is 2 g (x_i sum E - sum E y_j) in float32,
    so besides a relative part the difference has a floor of a few ulps of the terms that cancel."""
    floor = 4e-6 * max(xd.nan_to_num().abs().max().item(), yd.nan_to_num().abs().max().item())  # (padding may hold NaN)
    for a, b2, name in ((dx, dx2, "dx"), (dy, dy2, "dy")):
        for b in range(a.shape[0]):
            err = (a[b] - b2[b]).abs().max().item()
            assert err <= 2e-5 * a[b].abs().max().item() + floor, "%s of pair %d with and without E output: %g" % (name, b, err)


def check_against(ref, got, pairs=None, what=""):
    """ref: oracle dict over `pairs` (indices into the GPU batch), got: GPU dict over the batch."""
    B = ref["value"].shape[0]
    pairs = list(range(B)) if pairs is None else pairs
    for r, b in enumerate(pairs):
        v, w = got["value"][b], ref["value"][r]
        assert abs(v - w) <= VALUE_RTOL * max(abs(w), 1.0), "%s value pair %d: %r vs %r" % (what, b, v, w)
        for key in ("dx", "dy"):
            g, o = got[key][b], ref[key][r]
            scale = max(np.abs(o).max(), 1e-30)
            err = np.abs(g - o).max() / scale
            assert err <= GRAD_RTOL, "%s %s pair %d: rel err %.3e" % (what, key, b, err)
        if "E" in ref and "E" in got:
            err = np.abs(got["E"][b] - ref["E"][r]).max()
            assert err <= E_ATOL, "%s E pair %d: abs err %.3e" % (what, b, err)


# ------------------------------------------------------------------------------- hardware facts
def test_lane_shifts_behave_as_the_kernels_assume():
    out = binding.debug_lane_shift().cpu().numpy()
    np.testing.assert_array_equal(out[:64], np.concatenate([[-1], np.arange(63)]))
    np.testing.assert_array_equal(out[64:], np.concatenate([np.arange(1, 64), [-2]]))


# ------------------------------------------------------------------------------- intermediates
@pytest.mark.parametrize("B,N,M,D", [(2, 64, 64, 8), (3, 70, 45, 5), (2, 33, 130, 128), (1, 1, 1, 1)])
def test_unfused_cost_tensor(B, N, M, D):
    import torch

    say("cost tensor B=%d N=%d M=%d D=%d" % (B, N, M, D))
    x, y = workloads.normal_pairs(100 + N, B, N, M, D)
    xd, yd = to_dev(x), to_dev(y)
    _, desc, ws = pkg.sdtw_forward(xd, yd, 1.0, pkg.UNFUSED)
    d = binding.debug_export(desc, ws, binding.EXPORT_COST).cpu().numpy().astype(np.float64)
    torch.cuda.synchronize()
    ref = ((x[:, :, None, :].astype(np.float64) - y[:, None, :, :].astype(np.float64)) ** 2).sum(-1)
    for b in range(B):
        np.testing.assert_allclose(d[b], oracle.pair_tables(x[b], y[b], 1.0)["d"], rtol=0, atol=2e-5 * max(ref.max(), 1))
    np.testing.assert_allclose(d, ref, rtol=0, atol=2e-5 * max(ref.max(), 1))


@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("N,M,D,gamma", [(64, 64, 8, 1.0), (100, 77, 16, 0.1), (130, 31, 3, 0.5)])
def test_full_R_table(mode, N, M, D, gamma):
    import torch

    say("R table %s N=%d M=%d D=%d gamma=%g" % (mode, N, M, D, gamma))
    x, y = workloads.normal_pairs(200 + N, 2, N, M, D)
    xd, yd = to_dev(x), to_dev(y)
    value, desc, ws = pkg.sdtw_forward(xd, yd, gamma, MODES[mode])
    R = binding.debug_export(desc, ws, binding.EXPORT_R).cpu().numpy()
    torch.cuda.synchronize()
    for b in range(2):
        ref = oracle.pair_tables(x[b], y[b], gamma)["R"][1:N + 1, 1:M + 1]
        np.testing.assert_allclose(R[b], ref, rtol=1e-5, atol=1e-4)
        assert abs(value[b].item() - ref[-1, -1]) <= VALUE_RTOL * max(abs(ref[-1, -1]), 1)


# ------------------------------------------------------------------------------- end to end, small
SHAPES = [
    # B, N, M, D, gamma
    (4, 64, 64, 8, 1.0),       # config 1 shape
    (1, 1, 1, 4, 1.0),         # single cell
    (2, 1, 9, 3, 0.5),         # single row
    (2, 9, 1, 3, 0.5),         # single column
    (2, 2, 2, 2, 0.3),
    (3, 63, 33, 5, 0.1),       # ragged in both directions, odd D
    (3, 65, 31, 8, 0.1),
    (2, 64, 32, 12, 1.0),
    (2, 96, 160, 16, 0.1),     # N != M, several bands and macro-steps
    (2, 200, 129, 24, 0.01),   # small gamma, ragged tail in the last band and the last block
    (1, 257, 70, 128, 0.1),
    (2, 70, 90, 40, 0.2),      # D between the sizes the split operand copies are padded to
    (2, 66, 40, 72, 0.2),
]


@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma", SHAPES)
def test_value_E_and_gradients(mode, B, N, M, D, gamma):
    say("parity %s B=%d N=%d M=%d D=%d gamma=%g" % (mode, B, N, M, D, gamma))
    x, y = workloads.normal_pairs(300 + 7 * N + M, B, N, M, D)
    ref = oracle.batch(x, y, gamma, want_E=True)
    got = run_gpu(x, y, gamma, MODES[mode])
    check_against(ref, got, what="%s %s" % (mode, (B, N, M, D, gamma)))
    E = got["E"]
    assert np.all(np.isfinite(E)) and E.min() >= 0.0 and E.max() <= 1.0 + 1e-5
    np.testing.assert_allclose(E[:, -1, -1], 1.0, atol=1e-6)
    np.testing.assert_allclose(E[:, 0, 0], 1.0, atol=1e-4)


@pytest.mark.parametrize("shape", [1, 2, 4])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma", [(5, 200, 150, 16, 0.1), (2, 130, 257, 128, 0.05), (7, 65, 96, 20, 1.0),
                                           (3, 100, 90, 200, 0.5), (2, 300, 40, 8, 0.3), (3, 50, 70, 4, 1.0)])
def test_all_workgroup_shapes(shape, mode, B, N, M, D, gamma):
    # one band per workgroup, a chained pair of bands per workgroup (normally for 2 or more bands),
    # or 4 bands of 4 pairs (normally only for > 1536 band tasks): force each on small inputs
    # (odd numbers of bands, a single band, B not a multiple of 4, D above the register-operand
    # limit of 128 included)
    say("shape %d %s B=%d N=%d M=%d D=%d gamma=%g" % (shape, mode, B, N, M, D, gamma))
    x, y = workloads.normal_pairs(900 + N + D, B, N, M, D)
    ref = oracle.batch(x, y, gamma, want_E=True)
    binding.debug_force_workgroup_shape(shape)
    try:
        got = run_gpu(x, y, gamma, MODES[mode])
    finally:
        binding.debug_force_workgroup_shape(0)
    check_against(ref, got, what="shape %d %s" % (shape, mode))


@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("gamma", [0.01, 1.0, 50.0])
@pytest.mark.parametrize("kind", ["normal", "walk"])
@pytest.mark.parametrize("shape", [1, 2])
def test_alignment_only_looks_where_E_can_be_non_zero(shape, mode, gamma, kind):
    # 600 x 700: from 16 column blocks on the backward call of small problems first finds, per band,
    # the columns that can hold a non-zero E (from the boundary rows) and forms E only there.  Sparse
    # E (small gamma), dense E (gamma = 50: every cell non-zero) and both input recipes; E is compared
    # everywhere, so a block wrongly taken for zero would show.
    B, N, M, D = 3, 600, 700, 12
    x, y = (workloads.normal_pairs if kind == "normal" else workloads.walk_pairs)(77, B, N, M, D)
    # Both workgroup shapes of small problems: the look needs every band's edge rows in memory, also
    # those a chained pair hands over through LDS.
    say("alignment pruning shape %d %s gamma=%g %s" % (shape, mode, gamma, kind))
    ref = oracle.batch(x, y, gamma, want_E=True)
    binding.debug_force_workgroup_shape(shape)
    try:
        got = run_gpu(x, y, gamma, MODES[mode])
    finally:
        binding.debug_force_workgroup_shape(0)
    check_against(ref, got, what="alignment pruning %s gamma=%g %s" % (mode, gamma, kind))
    # float32 cannot hold anything the pruning may have dropped: wherever the oracle's E is above the
    # smallest normal float32 by a margin (the hardware exp2 flushes denormal results), the library's E is non-zero
    assert (got["E"][ref["E"] > 1e-36] > 0).all()


@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma", [(5, 200, 150, 16, 0.1), (2, 130, 257, 128, 0.05), (3, 64, 64, 8, 1.0),
                                           (2, 100, 90, 200, 0.5), (4, 300, 333, 33, 20.0), (1, 1, 1, 1, 1.0),
                                           (3, 31, 700, 64, 0.01)])
@pytest.mark.parametrize("pool", [-1, 0, 7])
def test_min_memory_flag(pool, mode, B, N, M, D, gamma):
    # SDTW_FLAG_MIN_MEMORY: small problems on the route of large ones with long sequences - checkpoints
    # instead of tables and (D <= 128) a compact E: only the non-zero 32x32 blocks, in a pool.  pool = 0 / 7:
    # a pool of that many blocks, which runs over, so that the backward call takes its second sweep, the
    # one that contracts every block of E into dx, dy where it stands.
    # Sparse to dense E, D that is no multiple of 32, D above 128 (a dense E stays in the workspace there).
    say("min memory %s B=%d N=%d M=%d D=%d gamma=%g pool=%d" % (mode, B, N, M, D, gamma, pool))
    x, y = workloads.normal_pairs(300 + N + D, B, N, M, D)
    ref = oracle.batch(x, y, gamma, want_E=True)
    binding.debug_set_pool_blocks(pool)
    try:
        got = run_gpu(x, y, gamma, MODES[mode], min_memory=True)
    finally:
        binding.debug_set_pool_blocks(-1)
    check_against(ref, got, what="min memory %s %dx%d" % (mode, N, M))
    plain = binding.make_desc(B, N, M, D, gamma, MODES[mode])
    assert pkg.sdtw_workspace_bytes(got["desc"]) < pkg.sdtw_workspace_bytes(plain) or N * M < 4096


@pytest.mark.parametrize("dtype", ["float16", "bfloat16"])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma,shape,min_memory", [
    (3, 200, 150, 16, 0.5, 0, False), (2, 130, 257, 128, 1.0, 0, False), (2, 100, 90, 200, 1.0, 0, False),
    (4, 300, 333, 33, 5.0, 0, True), (5, 96, 70, 64, 0.3, 1, False), (3, 260, 200, 128, 2.0, 4, False)])
def test_half_precision_inputs(dtype, mode, B, N, M, D, gamma, shape, min_memory):
    # float16 / bfloat16 sequences (Sec. 6, "Mixed precision"): the library's results are those of the
    # ROUNDED sequences, to the bars of the float32 entry points - the oracle gets the rounded values as
    # float32.  (The cost then takes one matrix-core product per 16 features instead of three.)
    import torch

    say("half inputs %s %s B=%d N=%d M=%d D=%d gamma=%g shape=%d min_memory=%s" % (dtype, mode, B, N, M, D, gamma, shape, min_memory))
    x, y = workloads.normal_pairs(700 + N + D, B, N, M, D)
    td = getattr(torch, dtype)
    xh, yh = torch.from_numpy(x).to(td).cuda(), torch.from_numpy(y).to(td).cuda()
    xr, yr = xh.float().cpu().numpy(), yh.float().cpu().numpy()
    ref = oracle.batch(xr, yr, gamma, want_E=True)
    binding.debug_force_workgroup_shape(shape)
    try:
        value, desc, ws = pkg.sdtw_forward_half(xh, yh, gamma, MODES[mode], min_memory=min_memory)
        dx, dy, _ = pkg.sdtw_backward_half(desc, ws)
        dx2, dy2, E = pkg.sdtw_backward_half(desc, ws, want_E=True)
        torch.cuda.synchronize()
    finally:
        binding.debug_force_workgroup_shape(0)
    assert binding.workspace_status(ws) == 0
    got = {"value": value.cpu().numpy().astype(np.float64), "dx": dx.cpu().numpy().astype(np.float64),
           "dy": dy.cpu().numpy().astype(np.float64), "E": E.cpu().numpy().astype(np.float64)}
    check_against(ref, got, what="half inputs %s %s" % (dtype, mode))
    assert_same_gradients(dx, dx2, dy, dy2, xh.float(), yh.float())
    # a workspace filled by the half entry point is not one of the float32 entry point
    with pytest.raises(pkg.SdtwError):
        pkg.sdtw_backward(desc, xh.float(), yh.float(), binding.Workspace(16))


def test_config1_tiny_oracle_case():
    wl = workloads.pair_workload("c1_tiny")
    say("config 1")
    ref = oracle.batch(wl.x, wl.y, wl.gamma, want_E=True)
    got = run_gpu(wl.x, wl.y, wl.gamma, pkg.UNFUSED)
    check_against(ref, got, what="c1")


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_zero_cost_gives_delannoy_table(mode):
    # data-free check at a size spanning bands: R[i,j] = -gamma log Del(i-1,j-1)
    import torch

    N, M, gamma = 150, 90, 1.0
    say("delannoy %s" % mode)
    x = np.full((1, N, 4), 0.5, dtype=np.float32)
    y = np.full((1, M, 4), 0.5, dtype=np.float32)
    value, desc, ws = pkg.sdtw_forward(to_dev(x), to_dev(y), gamma, MODES[mode])
    R = binding.debug_export(desc, ws, binding.EXPORT_R).cpu().numpy()[0]
    torch.cuda.synchronize()
    logdel = np.zeros((N, M))
    for i in range(1, N):
        for j in range(1, M):
            logdel[i, j] = np.logaddexp(np.logaddexp(logdel[i - 1, j], logdel[i, j - 1]), logdel[i - 1, j - 1])
    np.testing.assert_allclose(R, -gamma * logdel, rtol=1e-5, atol=1e-4)


@pytest.mark.parametrize("shape", [1, 4])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_zero_cost_alignment_matrix_is_the_delannoy_ratio(shape, mode):
    # identical constant sequences: every cost is 0, R is negative throughout and
    # E[i,j] = Del(i,j) Del(N-1-i, M-1-j) / Del(N-1, M-1) (0-based): nowhere near zero around the
    # diagonal, vanishing towards the far corners - also in the 4-band workgroups, whose backward
    # decides per macro-step whether E can be non-zero at all
    N, M, gamma = 200, 170, 1.0
    say("delannoy E shape %d %s" % (shape, mode))
    x = np.full((2, N, 4), 0.25, dtype=np.float32)
    y = np.full((2, M, 4), 0.25, dtype=np.float32)
    logdel = np.zeros((N, M))
    for i in range(1, N):
        for j in range(1, M):
            logdel[i, j] = np.logaddexp(np.logaddexp(logdel[i - 1, j], logdel[i, j - 1]), logdel[i - 1, j - 1])
    E_exact = np.exp(logdel + logdel[::-1, ::-1] - logdel[N - 1, M - 1])
    binding.debug_force_workgroup_shape(shape)
    try:
        got = run_gpu(x, y, gamma, MODES[mode])
    finally:
        binding.debug_force_workgroup_shape(0)
    assert np.abs(got["E"][0] - E_exact).max() <= E_ATOL
    assert np.abs(got["E"][1] - E_exact).max() <= E_ATOL
    assert abs(got["value"][0] + gamma * logdel[N - 1, M - 1]) <= 1e-4 * gamma * logdel[N - 1, M - 1]


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_upstream_gradient_and_shared_x(mode):
    say("grad_value / shared x %s" % mode)
    B, N, M, D, gamma = 3, 70, 50, 6, 0.2
    x, y = workloads.normal_pairs(77, B, N, M, D)
    gv = np.array([1.0, -2.0, 0.25])
    ref = oracle.batch(x, y, gamma, grad_value=gv)
    got = run_gpu(x, y, gamma, MODES[mode], grad_value=gv, want_E=False)
    check_against(ref, got, what="grad_value")
    ref = oracle.batch(x[0], y, gamma)
    got = run_gpu(x[0], y, gamma, MODES[mode], want_E=False)
    check_against(ref, got, what="shared x")


def test_fused_equals_unfused_to_rounding():
    x, y = workloads.normal_pairs(5, 4, 120, 140, 32)
    a = run_gpu(x, y, 0.1, pkg.UNFUSED)
    b = run_gpu(x, y, 0.1, pkg.FUSED)
    # (the two modes sum the squared norms in different orders: the costs differ by an ulp here and
    # there, 4e-6 at d ~ 64, which over gamma = 0.1 is a few 1e-5 relative in E)
    np.testing.assert_allclose(a["value"], b["value"], rtol=1e-6)
    np.testing.assert_allclose(a["E"], b["E"], atol=5e-5)
    np.testing.assert_allclose(a["dx"], b["dx"], atol=1e-4 * np.abs(a["dx"]).max())


def test_calls_run_on_the_callers_stream():
    # Two different problems enqueued on two side streams (default priority), nothing on the default
    # stream, no synchronisation until both are enqueued: each call's kernels must all be on its own
    # stream, or they would overtake the copies and each other.  Results as from one call at a time.
    import torch

    x1, y1 = workloads.normal_pairs(61, 6, 200, 170, 32)
    x2, y2 = workloads.normal_pairs(62, 3, 90, 310, 128)
    ref1 = oracle.batch(x1, y1, 0.1, want_E=False)
    ref2 = oracle.batch(x2, y2, 0.5, want_E=False)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    hx1, hy1, hx2, hy2 = (torch.from_numpy(a).pin_memory() for a in (x1, y1, x2, y2))
    out = {}
    for rep in range(3):
        with torch.cuda.stream(s1):
            xd1, yd1 = hx1.cuda(non_blocking=True), hy1.cuda(non_blocking=True)
            v1, d1, w1 = pkg.sdtw_forward(xd1, yd1, 0.1, pkg.FUSED)
            dx1, dy1, _ = pkg.sdtw_backward(d1, xd1, yd1, w1)
        with torch.cuda.stream(s2):
            xd2, yd2 = hx2.cuda(non_blocking=True), hy2.cuda(non_blocking=True)
            v2, d2, w2 = pkg.sdtw_forward(xd2, yd2, 0.5, pkg.UNFUSED)
            dx2, dy2, _ = pkg.sdtw_backward(d2, xd2, yd2, w2)
        s1.synchronize()
        s2.synchronize()
        assert binding.workspace_status(w1) == 0 and binding.workspace_status(w2) == 0
        out[rep] = [t.cpu().numpy().astype(np.float64) for t in (v1, dx1, dy1, v2, dx2, dy2)]
        check_against(ref1, {"value": out[rep][0], "dx": out[rep][1], "dy": out[rep][2]}, what="stream 1")
        check_against(ref2, {"value": out[rep][3], "dx": out[rep][4], "dy": out[rep][5]}, what="stream 2")
    for a, b in zip(out[0], out[2]):
        np.testing.assert_array_equal(a, b)  # and the same bits every time


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_forward_and_backward_replay_from_a_captured_graph(mode):
    # The entry points only launch kernels (no allocation, no memset, no synchronisation), so a
    # forward + backward pair can be captured into a graph once and replayed on new inputs.  Every
    # replay is compared with the same calls made eagerly, with eager work between the replays.
    import torch

    B, N, M, D, gamma = 5, 150, 130, 16, 0.2
    xs, ys = torch.empty(B, N, D, device="cuda"), torch.empty(B, M, D, device="cuda")
    value = torch.empty(B, device="cuda")
    dx, dy = torch.empty(B, N, D, device="cuda"), torch.empty(B, M, D, device="cuda")
    x0, y0 = workloads.normal_pairs(70, B, N, M, D)
    xs.copy_(to_dev(x0)); ys.copy_(to_dev(y0))
    _, desc, ws = pkg.sdtw_forward(xs, ys, gamma, MODES[mode], value=value)  # warm-up, allocates the workspace
    pkg.sdtw_backward(desc, xs, ys, ws, dx=dx, dy=dy)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pkg.sdtw_forward(xs, ys, gamma, MODES[mode], workspace=ws, value=value)
        pkg.sdtw_backward(desc, xs, ys, ws, dx=dx, dy=dy)
    for rep in range(4):
        x, y = workloads.normal_pairs(71 + rep, B, N, M, D)
        xe, ye = to_dev(x), to_dev(y)
        ve, de, we = pkg.sdtw_forward(xe, ye, gamma, MODES[mode])  # eager, other buffers
        dxe, dye, _ = pkg.sdtw_backward(de, xe, ye, we)
        xs.copy_(xe); ys.copy_(ye)
        graph.replay()
        torch.cuda.synchronize()
        assert binding.workspace_status(ws) == 0
        assert torch.equal(value, ve) and torch.equal(dx, dxe) and torch.equal(dy, dye), "replay %d" % rep
    ref = oracle.batch(x, y, gamma, want_E=False)
    check_against(ref, {"value": value.cpu().numpy().astype(np.float64), "dx": dx.cpu().numpy().astype(np.float64),
                        "dy": dy.cpu().numpy().astype(np.float64)}, what="graph %s" % mode)


def test_symmetry():
    x, y = workloads.normal_pairs(6, 2, 90, 75, 8)
    a = run_gpu(x, y, 0.5, pkg.FUSED)
    b = run_gpu(y, x, 0.5, pkg.FUSED)
    np.testing.assert_allclose(a["value"], b["value"], rtol=1e-6)
    np.testing.assert_allclose(a["E"], np.swapaxes(b["E"], 1, 2), atol=1e-5)
    np.testing.assert_allclose(a["dx"], b["dy"], atol=1e-4 * np.abs(a["dx"]).max())


def test_value_only_forward_matches_and_refuses_backward():
    import torch

    x, y = workloads.normal_pairs(11, 3, 150, 170, 12)
    xd, yd = to_dev(x), to_dev(y)
    ref = oracle.batch(x, y, 0.2, backward=False)
    for mode in (pkg.UNFUSED, pkg.FUSED):
        value, desc, ws = pkg.sdtw_forward(xd, yd, 0.2, mode, value_only=True)
        torch.cuda.synchronize()
        assert binding.workspace_status(ws) == 0
        np.testing.assert_allclose(value.cpu().numpy(), ref["value"], rtol=VALUE_RTOL)
        full = pkg.sdtw_workspace_bytes(binding.make_desc(3, 150, 170, 12, 0.2, mode))
        assert ws.nbytes < full
        with pytest.raises(pkg.SdtwError) as err:
            pkg.sdtw_backward(desc, xd, yd, ws)
        assert err.value.status == binding.STATUS_STATE


def test_backward_twice_after_one_forward_gives_the_same_result():
    import torch

    x, y = workloads.normal_pairs(12, 2, 100, 130, 8)
    xd, yd = to_dev(x), to_dev(y)
    for shape in (1, 2, 4):
        binding.debug_force_workgroup_shape(shape)
        try:
            _, desc, ws = pkg.sdtw_forward(xd, yd, 0.3, pkg.FUSED)
            dx1, dy1, _ = pkg.sdtw_backward(desc, xd, yd, ws)
            dx2, dy2, _ = pkg.sdtw_backward(desc, xd, yd, ws)
            torch.cuda.synchronize()
        finally:
            binding.debug_force_workgroup_shape(0)
        assert binding.workspace_status(ws) == 0
        assert torch.equal(dx1, dx2) and torch.equal(dy1, dy2)

@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma,scale", [
    (2, 1, 5000, 8, 0.1, 1.0),        # a single row, 157 macro-steps
    (2, 5000, 1, 8, 0.1, 1.0),        # a single column, 79 bands
    (1, 3000, 7, 1, 1.0, 1.0),        # one feature
    (2, 200, 200, 16, 1e-3, 1.0),     # gamma far below the costs: E is a single path
    (2, 200, 200, 16, 100.0, 1.0),    # gamma far above them: E spreads over the whole grid
    (2, 128, 128, 128, 0.1, 100.0),   # inputs of magnitude 100 (costs ~ 2.5e6) ...
    (2, 128, 128, 128, 0.1, 1e-3),    # ... and of magnitude 0.001
    (70, 64, 64, 128, 0.1, 1.0),      # more pairs than fit one round of workgroups of a band
])
def test_extreme_shapes_and_magnitudes(mode, B, N, M, D, gamma, scale):
    say("extreme %s B=%d N=%d M=%d D=%d gamma=%g scale=%g" % (mode, B, N, M, D, gamma, scale))
    x, y = workloads.normal_pairs(777 + N + M + D, B, N, M, D)
    x, y = (x * scale).astype(np.float32), (y * scale).astype(np.float32)
    ref = oracle.batch(x, y, gamma, want_E=False)
    got = run_gpu(x, y, gamma, MODES[mode], want_E=False)
    check_against(ref, got, what="extreme %s" % mode)
    assert np.all(np.isfinite(got["dx"])) and np.all(np.isfinite(got["dy"]))


@pytest.mark.parametrize("ragged", [False, True])
@pytest.mark.parametrize("N,M", [(33, 257), (97, 288), (64, 289), (130, 320), (65, 321), (32, 225)])
def test_alignment_at_the_row_length_limits(N, M, ragged):
    # Small problems with up to 10 column blocks form E per block row with the whole row in LDS,
    # longer rows in runs of blocks per wavefront: the last lengths of the one (M = 320), the first
    # of the other (321), rows that end one past a block (257, 289: the sweep then has one macro-step
    # fewer beyond the last block), and band counts that leave half a band empty (N = 33, 97, 32)
    say("row limits N=%d M=%d ragged=%s" % (N, M, ragged))
    B, D, gamma = 3, 8, 0.3
    x, y = workloads.normal_pairs(4100 + N + M, B, N, M, D)
    if ragged:
        xl = workloads.ragged_lengths(5 + N, B, N)
        yl = workloads.ragged_lengths(6 + M, B, M, shortest=M - 40)[::-1].copy()
        ref = oracle.ragged_batch(x, y, xl, yl, gamma, want_E=True)
        got = run_gpu_ragged(x, y, xl, yl, gamma, MODES["fused"])
        for b in range(B):
            assert not got["E"][b, xl[b]:].any() and not got["E"][b, :, yl[b]:].any()
    else:
        ref = oracle.batch(x, y, gamma, want_E=True)
        got = run_gpu(x, y, gamma, MODES["fused"])
    check_against(ref, got, what="row limits %d x %d" % (N, M))


# ------------------------------------------------------------------------------- ragged batches
def run_gpu_ragged(x, y, xl, yl, gamma, mode, grad_value=None, want_E=True, min_memory=False):
    import torch

    xd, yd = to_dev(x), to_dev(y)
    xld = to_dev(xl) if xl is not None else None
    yld = to_dev(yl) if yl is not None else None
    value, desc, ws = pkg.sdtw_forward_ragged(xd, yd, xld, yld, gamma, mode, min_memory=min_memory)
    gv = to_dev(grad_value.astype(np.float32)) if grad_value is not None else None
    return ragged_backward_both_routes(value, desc, ws, xd, yd, xld, yld, gv, want_E)


def ragged_backward_both_routes(value, desc, ws, xd, yd, xld, yld, gv, want_E):
    """Gradients from the backward call without E output, E from a second call (see run_gpu)."""
    import torch

    dx, dy, _ = pkg.sdtw_backward_ragged(desc, xd, yd, xld, yld, ws, grad_value=gv)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    out = {"value": value.cpu().numpy().astype(np.float64), "dx": dx.cpu().numpy().astype(np.float64),
           "dy": dy.cpu().numpy().astype(np.float64)}
    if want_E:
        dx2, dy2, E = pkg.sdtw_backward_ragged(desc, xd, yd, xld, yld, ws, grad_value=gv, want_E=True)
        torch.cuda.synchronize()
        assert binding.workspace_status(ws) == 0
        out["E"] = E.cpu().numpy().astype(np.float64)
        assert_same_gradients(dx, dx2, dy, dy2, xd, yd)
    return out


@pytest.mark.parametrize("shape", [0, 1, 2, 4])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma", [(6, 200, 150, 16, 0.1), (4, 130, 257, 128, 0.05), (5, 64, 64, 8, 1.0),
                                           (3, 300, 90, 200, 0.5)])
def test_ragged_batches(shape, mode, B, N, M, D, gamma):
    # every pair with lengths of its own (pair 0 full, the last pair of length 1 on the x side and
    # full on the y side or the reverse), in each workgroup shape; E and gradients beyond the lengths
    # must come out as exact zeros
    say("ragged shape %d %s B=%d N=%d M=%d D=%d" % (shape, mode, B, N, M, D))
    x, y = workloads.normal_pairs(300 + N + D, B, N, M, D)
    xl = workloads.ragged_lengths(31 + N, B, N)
    yl = workloads.ragged_lengths(32 + M, B, M)[::-1].copy()
    gv = np.linspace(0.5, 2.0, B)
    ref = oracle.ragged_batch(x, y, xl, yl, gamma, grad_value=gv, want_E=True)
    binding.debug_force_workgroup_shape(shape)
    try:
        got = run_gpu_ragged(x, y, xl, yl, gamma, MODES[mode], grad_value=gv)
    finally:
        binding.debug_force_workgroup_shape(0)
    check_against(ref, got, what="ragged shape %d %s" % (shape, mode))
    for b in range(B):
        assert not got["E"][b, xl[b]:].any() and not got["E"][b, :, yl[b]:].any()
        assert not got["dx"][b, xl[b]:].any() and not got["dy"][b, yl[b]:].any()


@pytest.mark.parametrize("pool", [-1, 3])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("w", [0, 70])
def test_compact_E_with_lengths_and_band(w, mode, pool):
    # per-pair lengths (NaN in the padding) and a band constraint on the compact layout, through the pool
    # and - pool of 3 blocks - through the second, contracting sweep, which masks by the lengths itself
    B, N, M, D, gamma = 5, 260, 230, 24, 0.2
    say("compact E ragged w=%d %s pool=%d" % (w, mode, pool))
    x, y = workloads.normal_pairs(911, B, N, M, D)
    xl = workloads.ragged_lengths(41, B, N, shortest=200)
    yl = workloads.ragged_lengths(42, B, M, shortest=200)[::-1].copy()
    for b in range(B):
        x[b, xl[b]:] = np.nan
        y[b, yl[b]:] = np.nan
    gv = np.linspace(0.5, 2.0, B)
    ref = oracle.ragged_batch(np.nan_to_num(x), np.nan_to_num(y), xl, yl, gamma, grad_value=gv, want_E=True,
                              bandwidth=w if w else None)
    binding.debug_set_pool_blocks(pool)
    try:
        if w:
            got = run_gpu_band(x, y, gamma, MODES[mode], w, xl=xl, yl=yl, min_memory=True)
        else:
            got = run_gpu_ragged(x, y, xl, yl, gamma, MODES[mode], grad_value=gv, min_memory=True)
    finally:
        binding.debug_set_pool_blocks(-1)
    if w:  # (the band helper takes no upstream gradient)
        ref = oracle.ragged_batch(np.nan_to_num(x), np.nan_to_num(y), xl, yl, gamma, want_E=True, bandwidth=w)
    check_against(ref, got, what="compact E ragged w=%d %s pool=%d" % (w, mode, pool))
    for b in range(B):
        assert not got["dx"][b, xl[b]:].any() and not got["dy"][b, yl[b]:].any()


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_ragged_results_do_not_depend_on_the_padding(mode):
    import torch

    B, N, M, D, gamma = 4, 150, 210, 12, 0.2
    x, y = workloads.normal_pairs(81, B, N, M, D)
    xl = workloads.ragged_lengths(82, B, N, shortest=3)
    yl = workloads.ragged_lengths(83, B, M, shortest=70)
    a = run_gpu_ragged(x, y, xl, yl, gamma, MODES[mode])
    x2, y2 = x.copy(), y.copy()
    for b in range(B):
        x2[b, xl[b]:] = 1e4
        y2[b, yl[b]:] = np.nan
    c = run_gpu_ragged(x2, y2, xl, yl, gamma, MODES[mode])
    for key in ("value", "dx", "dy", "E"):
        assert np.array_equal(a[key], c[key]), key
    # one length vector only, and none at all (then the plain entry point's result, bit for bit)
    ref = oracle.ragged_batch(x, y, None, yl, gamma, want_E=True)
    check_against(ref, run_gpu_ragged(x, y, None, yl, gamma, MODES[mode]), what="y lengths only")
    plain = run_gpu(x, y, gamma, MODES[mode])
    none = run_gpu_ragged(x, y, None, None, gamma, MODES[mode])
    for key in ("value", "dx", "dy", "E"):
        assert np.array_equal(plain[key], none[key]), key
    torch.cuda.synchronize()


def test_ragged_large_regime_and_state_check():
    import torch

    # more than 1536 band tasks: 4-band workgroups, recomputing backward in both modes
    B, N, M, D, gamma = 72, 1500, 400, 24, 0.2
    say("ragged, large regime B=%d N=%d M=%d" % (B, N, M))
    x, y = workloads.normal_pairs(52, B, N, M, D)
    xl = workloads.ragged_lengths(53, B, N)
    yl = workloads.ragged_lengths(54, B, M)
    pairs = [0, 1, 20, 47]
    ref = oracle.ragged_batch(x[pairs], y[pairs], xl[pairs], yl[pairs], gamma)
    for mode in ("unfused", "fused"):
        got = run_gpu_ragged(x, y, xl, yl, gamma, MODES[mode], want_E=False)
        check_against(ref, got, pairs=pairs, what="ragged large " + mode)
        for b in range(B):
            assert not got["dx"][b, xl[b]:].any() and not got["dy"][b, yl[b]:].any()
    # a backward call with other length vectors than the forward's is refused on the device
    xd, yd, xld, yld = to_dev(x[:2, :100]), to_dev(y[:2, :90]), to_dev(xl[:2] % 100 + 1), to_dev(yl[:2] % 90 + 1)
    _, desc, ws = pkg.sdtw_forward_ragged(xd, yd, xld, yld, gamma, pkg.FUSED)
    other = xld.clone()
    dx, dy, _ = pkg.sdtw_backward_ragged(desc, xd, yd, other, yld, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == binding.STATUS_STATE
    assert torch.isnan(dx).all() and torch.isnan(dy).all()
    _, desc, ws = pkg.sdtw_forward_ragged(xd, yd, xld, yld, gamma, pkg.FUSED)
    dx, dy, _ = pkg.sdtw_backward(desc, xd, yd, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == binding.STATUS_STATE


# ------------------------------------------------------------------------------- band constraint |i-j| <= w
def run_gpu_band(x, y, gamma, mode, w, want_E=True, xl=None, yl=None, min_memory=False):
    import torch

    xd, yd = to_dev(x), to_dev(y)
    xld = to_dev(xl) if xl is not None else None
    yld = to_dev(yl) if yl is not None else None
    value, desc, ws = pkg.sdtw_forward_ragged(xd, yd, xld, yld, gamma, mode, bandwidth=w, min_memory=min_memory)
    return ragged_backward_both_routes(value, desc, ws, xd, yd, xld, yld, None, want_E)


BAND_CASES = [
    (3, 200, 150, 16, 0.1, (50, 64, 97, 400)),       # w = |N-M| is the narrowest band that holds the last cell
    (2, 130, 257, 128, 0.05, (127, 160)),
    (4, 300, 300, 8, 1.0, (1, 5, 31, 32, 33, 63, 64, 65, 100)),
    (3, 64, 64, 4, 0.5, (1, 63)),
    (2, 100, 90, 200, 0.5, (20,)),                    # D above the register-operand limit
    (5, 500, 520, 40, 0.2, (20, 77)),
]


@pytest.mark.parametrize("shape", [0, 1, 2, 4])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma,widths", BAND_CASES)
def test_band_constraint(shape, mode, B, N, M, D, gamma, widths):
    x, y = workloads.normal_pairs(700 + N + D, B, N, M, D)
    ii, jj = np.indices((N, M))
    for w in widths:
        say("band w=%d shape %d %s B=%d N=%d M=%d D=%d" % (w, shape, mode, B, N, M, D))
        ref = oracle.batch(x, y, gamma, want_E=True, bandwidth=w)
        binding.debug_force_workgroup_shape(shape)
        try:
            got = run_gpu_band(x, y, gamma, MODES[mode], w)
        finally:
            binding.debug_force_workgroup_shape(0)
        check_against(ref, got, what="band %d shape %d %s" % (w, shape, mode))
        assert not got["E"][:, np.abs(ii - jj) > w].any()


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_band_constraint_long_and_narrow(mode):
    # the sweeps skip most macro-steps of every band; small regime
    B, N, M, D, gamma, w = 3, 4096, 4000, 8, 0.1, 130
    say("band long %s" % mode)
    x, y = workloads.walk_pairs(61, B, N, M, D)
    ref = oracle.batch(x, y, gamma, bandwidth=w)
    got = run_gpu_band(x, y, gamma, MODES[mode], w, want_E=False)
    check_against(ref, got, what="band long " + mode)


def test_band_constraint_large_regime_ragged_and_state_check():
    import torch

    # more than 1536 band tasks would be: 4-band workgroups, recomputing backward in both modes;
    # per-pair lengths whose difference stays inside the band
    B, N, M, D, gamma, w = 44, 1600, 1500, 24, 0.2, 230
    say("band, large regime B=%d N=%d M=%d w=%d" % (B, N, M, w))
    x, y = workloads.normal_pairs(71, B, N, M, D)
    xl = workloads.ragged_lengths(72, B, N, shortest=1300)
    yl = np.minimum(M, np.maximum(1, xl + workloads.ragged_lengths(73, B, 2 * w, shortest=0) - w)).astype(np.int32)
    assert (np.abs(xl - yl) <= w).all()
    pairs = [0, 9, 43]
    ii, jj = np.indices((N, M))
    for mode in ("unfused", "fused"):
        ref = oracle.batch(x[pairs], y[pairs], gamma, want_E=True, bandwidth=w)
        ref_r = oracle.ragged_batch(x[pairs], y[pairs], xl[pairs], yl[pairs], gamma, bandwidth=w)
        # as the library would run it (few bands of a pair are busy at a time: one band per workgroup)
        # and in the 4-band workgroups of large problems
        for shape in (0, 4):
            binding.debug_force_workgroup_shape(shape)
            try:
                got = run_gpu_band(x, y, gamma, MODES[mode], w)
                got_r = run_gpu_band(x, y, gamma, MODES[mode], w, want_E=False, xl=xl, yl=yl)
            finally:
                binding.debug_force_workgroup_shape(0)
            check_against(ref, got, pairs=pairs, what="band large %s shape %d" % (mode, shape))
            assert not got["E"][:, np.abs(ii - jj) > w].any()
            check_against(ref_r, got_r, pairs=pairs, what="band large ragged %s shape %d" % (mode, shape))
    # a backward call with another bandwidth than the forward's is refused on the device
    xd, yd = to_dev(x[:2, :100]), to_dev(y[:2, :90])
    _, desc, ws = pkg.sdtw_forward(xd, yd, gamma, pkg.FUSED, bandwidth=30)
    desc.bandwidth = 31
    dx, dy, _ = pkg.sdtw_backward(desc, xd, yd, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == binding.STATUS_STATE
    assert torch.isnan(dx).all() and torch.isnan(dy).all()


# ------------------------------------------------------------------------------- random configurations
@pytest.mark.parametrize("seed", range(24))
def test_random_configurations(seed):
    # shapes, gamma, mode, band, per-pair lengths and workgroup shape drawn at random (seeded): every
    # option of the plain and ragged entry points in combination
    rng = np.random.default_rng(4000 + seed)
    B = int(rng.integers(1, 7))
    N = int(rng.integers(1, 330))
    M = int(rng.integers(1, 330))
    D = int(rng.choice([1, 3, 8, 16, 20, 33, 64, 100, 128, 150]))
    gamma = float(rng.choice([0.02, 0.1, 0.5, 1.0, 3.0]))
    mode = str(rng.choice(["unfused", "fused"]))
    shape = int(rng.choice([0, 0, 1, 2, 4]))
    ragged = bool(rng.integers(0, 2))
    banded = bool(rng.integers(0, 2))
    x, y = workloads.normal_pairs(5000 + seed, B, N, M, D)
    xl = yl = None
    w = 0
    if ragged:
        xl = workloads.ragged_lengths(6000 + seed, B, N)
        yl = workloads.ragged_lengths(7000 + seed, B, M)
    if banded:
        diff = int(np.abs((xl if ragged else N) - (yl if ragged else M)).max())
        w = max(1, diff + int(rng.integers(0, 40)))
    say("random %d: B=%d N=%d M=%d D=%d gamma=%g %s shape=%d ragged=%d w=%d" % (seed, B, N, M, D, gamma, mode, shape, ragged, w))
    ref = oracle.ragged_batch(x, y, xl, yl, gamma, want_E=True, bandwidth=w if banded else None)
    binding.debug_force_workgroup_shape(shape)
    try:
        got = run_gpu_band(x, y, gamma, MODES[mode], w, xl=xl, yl=yl)
    finally:
        binding.debug_force_workgroup_shape(0)
    check_against(ref, got, what="random %d" % seed)


# ------------------------------------------------------------------------------- normalised Soft-DTW
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma,shared", [(3, 40, 40, 8, 0.5, False), (2, 130, 75, 16, 0.1, False),
                                                  (4, 70, 200, 12, 1.0, True),
                                                  # equal lengths, nothing shared: the three terms as one batch
                                                  # (several bands, a ragged last block, D not a multiple of 4 / of 16)
                                                  (5, 150, 150, 21, 0.2, False), (7, 257, 257, 128, 0.1, False),
                                                  (2, 1, 1, 4, 1.0, False), (3, 2, 2, 3, 0.5, False),
                                                  # equal lengths but a shared x: three passes
                                                  (3, 96, 96, 8, 0.5, True)])
@pytest.mark.parametrize("min_memory", [False, True])
def test_normalized_value_and_gradients(min_memory, mode, B, N, M, D, gamma, shared):
    import torch

    say("normalised %s B=%d N=%d M=%d D=%d gamma=%g shared_x=%s min_memory=%s" % (mode, B, N, M, D, gamma, shared, min_memory))
    x, y = workloads.normal_pairs(700 + N, B, N, M, D)
    if shared:
        x = x[0]
    gv = np.linspace(0.5, 2.0, B)
    ref = oracle.normalized(np.broadcast_to(x, (B, N, D)) if shared else x, y, gamma, grad_value=gv)
    plain = oracle.batch(x, y, gamma, grad_value=gv)  # scale of the terms that cancel
    xd, yd = to_dev(x), to_dev(y)
    value, desc, ws = pkg.sdtw_normalized_forward(xd, yd, gamma, MODES[mode], min_memory=min_memory)
    dx, dy = pkg.sdtw_normalized_backward(desc, xd, yd, ws, grad_value=to_dev(gv.astype(np.float32)))
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    v = value.cpu().numpy().astype(np.float64)
    for b in range(B):
        scale = max(np.abs(ref["parts"][:, b]).max(), 1.0)
        assert abs(v[b] - ref["value"][b]) <= VALUE_RTOL * scale, (b, v[b], ref["value"][b])
    for got, key in ((dx, "dx"), (dy, "dy")):
        g = got.cpu().numpy().astype(np.float64)
        for b in range(B):
            scale = np.abs(plain[key][b]).max()
            assert np.abs(g[b] - ref[key][b]).max() <= GRAD_RTOL * scale, (key, b)


def test_normalized_batch_gives_one_gradient_alone():
    # the one-batch path with only dx or only dy asked for: same values as with both
    import torch

    x, y = workloads.normal_pairs(21, 4, 100, 100, 16)
    xd, yd = to_dev(x), to_dev(y)
    value, desc, ws = pkg.sdtw_normalized_forward(xd, yd, 0.3, pkg.FUSED)
    dx, dy = pkg.sdtw_normalized_backward(desc, xd, yd, ws)
    dx1, none1 = pkg.sdtw_normalized_backward(desc, xd, yd, ws, want_dy=False)
    none2, dy2 = pkg.sdtw_normalized_backward(desc, xd, yd, ws, want_dx=False)
    torch.cuda.synchronize()
    assert none1 is None and none2 is None
    assert torch.equal(dx, dx1) and torch.equal(dy, dy2)


def test_normalized_calls_replay_from_a_captured_graph():
    # the one-batch path (gather, forward, combine; backward, combine) captured once, replayed on new inputs
    import torch

    B, N, D, gamma = 4, 120, 16, 0.3
    xs, ys = torch.empty(B, N, D, device="cuda"), torch.empty(B, N, D, device="cuda")
    value = torch.empty(B, device="cuda")
    dx, dy = torch.empty(B, N, D, device="cuda"), torch.empty(B, N, D, device="cuda")
    x0, y0 = workloads.normal_pairs(80, B, N, N, D)
    xs.copy_(to_dev(x0)); ys.copy_(to_dev(y0))
    _, desc, ws = pkg.sdtw_normalized_forward(xs, ys, gamma, pkg.FUSED, value=value)
    pkg.sdtw_normalized_backward(desc, xs, ys, ws, dx=dx, dy=dy)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pkg.sdtw_normalized_forward(xs, ys, gamma, pkg.FUSED, workspace=ws, value=value)
        pkg.sdtw_normalized_backward(desc, xs, ys, ws, dx=dx, dy=dy)
    for rep in range(3):
        x, y = workloads.normal_pairs(81 + rep, B, N, N, D)
        xe, ye = to_dev(x), to_dev(y)
        ve, de, we = pkg.sdtw_normalized_forward(xe, ye, gamma, pkg.FUSED)
        dxe, dye = pkg.sdtw_normalized_backward(de, xe, ye, we)
        xs.copy_(xe); ys.copy_(ye)
        graph.replay()
        torch.cuda.synchronize()
        assert binding.workspace_status(ws) == 0
        assert torch.equal(value, ve) and torch.equal(dx, dxe) and torch.equal(dy, dye), "replay %d" % rep


def test_normalized_of_identical_sequences_is_zero():
    import torch

    x, _ = workloads.normal_pairs(15, 3, 90, 90, 8)
    xd = to_dev(x)
    value, desc, ws = pkg.sdtw_normalized_forward(xd, xd, 0.3, pkg.FUSED)
    dx, dy = pkg.sdtw_normalized_backward(desc, xd, xd, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    assert torch.all(value.abs() <= 1e-3)
    assert torch.all((dx + dy).abs() <= 1e-3 * max(dx.abs().max().item(), 1.0))


# ------------------------------------------------------------------------------- device-side errors
def test_backward_without_forward_is_refused_on_the_device():
    import torch

    x, y = workloads.normal_pairs(8, 2, 40, 40, 4)
    xd, yd = to_dev(x), to_dev(y)
    desc = binding.make_desc(2, 40, 40, 4, 1.0, pkg.FUSED)
    ws = binding.Workspace(pkg.sdtw_workspace_bytes(desc))
    ws.buffer.zero_()
    dx, dy, E = pkg.sdtw_backward(desc, xd, yd, ws, want_E=True)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == binding.STATUS_STATE
    assert torch.isnan(dx).all() and torch.isnan(dy).all() and torch.isnan(E).all()
    # a forward for another descriptor does not make it valid either
    pkg.sdtw_forward(xd, yd, 0.5, pkg.FUSED, workspace=ws)
    dx, dy, _ = pkg.sdtw_backward(desc, xd, yd, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == binding.STATUS_STATE and torch.isnan(dx).all()
    # the matching forward does
    _, d2, _ = pkg.sdtw_forward(xd, yd, 1.0, pkg.FUSED, workspace=ws)
    dx, dy, _ = pkg.sdtw_backward(d2, xd, yd, ws)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0 and torch.isfinite(dx).all()


def test_a_band_that_cannot_wait_gives_up_instead_of_hanging():
    import torch

    x, y = workloads.normal_pairs(9, 8, 512, 512, 8)
    xd, yd = to_dev(x), to_dev(y)
    binding.debug_set_spin_limit(0)
    try:
        value, desc, ws = pkg.sdtw_forward(xd, yd, 1.0, pkg.FUSED)
        torch.cuda.synchronize()
        status = binding.workspace_status(ws)
    finally:
        binding.debug_set_spin_limit(1 << 23)
    # either every band happened to find its neighbour ready, or the timeout was recorded;
    # in both cases every kernel has exited
    assert status in (0, binding.STATUS_TIMEOUT)
    value, desc, ws = pkg.sdtw_forward(xd, yd, 1.0, pkg.FUSED)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    ref = oracle.batch(x[:2], y[:2], 1.0, backward=False)
    np.testing.assert_allclose(value[:2].cpu().numpy(), ref["value"], rtol=VALUE_RTOL)


# ------------------------------------------------------------------------------- rectangular at scale
@pytest.mark.parametrize("mode", ["unfused", "fused"])
@pytest.mark.parametrize("B,N,M,D,gamma", [(3, 4096, 320, 32, 0.1), (3, 200, 5000, 16, 0.05)])
def test_rectangular_at_scale(mode, B, N, M, D, gamma):
    # N != M well beyond one band / a few macro-steps in either direction (Sec. 5 allows unequal
    # lengths; the paper only times squares).  The alignment hugs one side for most of its length.
    say("rectangular %s B=%d N=%d M=%d D=%d gamma=%g" % (mode, B, N, M, D, gamma))
    x, y = workloads.walk_pairs(40 + N % 7, B, N, M, D)
    ref = oracle.batch(x, y, gamma)
    got = run_gpu(x, y, gamma, MODES[mode], want_E=False)
    check_against(ref, got, what="rectangular %s %dx%d" % (mode, N, M))


def test_rectangular_large_regime():
    # more than 1536 band tasks with N != M: the 4-band workgroups, recomputing backward
    B, N, M, D, gamma = 64, 1700, 300, 24, 0.2
    say("rectangular, large regime B=%d N=%d M=%d" % (B, N, M))
    x, y = workloads.normal_pairs(51, B, N, M, D)
    pairs = [0, 17, 39]
    for gamma in (0.2, 0.01, 20.0):
        # sparse to dense E: the recomputing backward skips the macro-steps whose E it can prove to be
        # zero (most of them at gamma = 0.01, none at gamma = 20); E itself is compared everywhere
        ref = oracle.batch(x[pairs], y[pairs], gamma, want_E=True)
        for mode in ("unfused", "fused"):
            got = run_gpu(x, y, gamma, MODES[mode], want_E=True)
            check_against(ref, got, pairs=pairs, what="rectangular large %s gamma=%g" % (mode, gamma))
            for r, b in enumerate(pairs):
                assert (got["E"][b][ref["E"][r] > 1e-36] > 0).all()


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_many_bands_few_pairs(mode):
    # 512 bands per pair and a batch that does not fill the last 4-band workgroup (B = 5: one workgroup
    # in two runs with three idle slots); every band after the first hangs on a chain of 511 hand-overs
    B, N, M, D, gamma = 5, 32768, 600, 8, 0.5
    say("many bands %s B=%d N=%d M=%d" % (mode, B, N, M))
    x, y = workloads.walk_pairs(73, B, N, M, D)
    pairs = [0, 4]
    ref = oracle.batch(x[pairs], y[pairs], gamma, nthreads=2)
    got = run_gpu(x, y, gamma, MODES[mode], want_E=False)
    check_against(ref, got, pairs=pairs, what="many bands " + mode)
    assert np.all(np.isfinite(got["dx"])) and np.all(np.isfinite(got["dy"]))


# ------------------------------------------------------------------------------- benchmark configurations
@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_config2_full(mode):
    wl = workloads.pair_workload("c2_b32_l256")
    say("config 2 %s" % mode)
    ref = oracle.batch(wl.x, wl.y, wl.gamma)
    got = run_gpu(wl.x, wl.y, wl.gamma, MODES[mode], want_E=False)
    check_against(ref, got, what="c2 " + mode)


# E has no bar of its own in the task.  Its error is that of the float32 cost: d is off by about
# eps32 * (||x||^2 + ||y||^2) per cell, which moves the exponent of the weight of an alignment by that
# over gamma for every cell in which two competing alignments differ (a handful of cells, since
# longer detours are exponentially suppressed), and E(1 - E) <= 1/4 turns a relative weight error into
# an absolute error of E.  With eps32 = 6e-8 and four differing cells:
def e_tolerance(x, y, gamma):
    norms = float((x.astype(np.float64) ** 2).sum(-1).mean() + (y.astype(np.float64) ** 2).sum(-1).mean())
    return max(E_ATOL, 0.25 * 2.0 * 6e-8 * norms / gamma)


@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_config3_full_size_sampled_pairs(mode):
    wl = workloads.pair_workload("c3_b32_l1024_walk")
    say("config 3 %s" % mode)
    pairs = [0, 13, 31]
    ref = oracle.batch(wl.x[pairs], wl.y[pairs], wl.gamma, want_E=True)
    got = run_gpu(wl.x, wl.y, wl.gamma, MODES[mode], want_E=True)
    check_against({k: v for k, v in ref.items() if k != "E"}, got, pairs=pairs, what="c3 " + mode)
    assert np.all(np.isfinite(got["dx"])) and np.all(np.isfinite(got["dy"]))
    # the whole alignment matrix of the sampled pairs, through the E output of the backward call
    tol = e_tolerance(wl.x[pairs], wl.y[pairs], wl.gamma)
    for r, b in enumerate(pairs):
        err = np.abs(got["E"][b] - ref["E"][r]).max()
        say("  c3 %s pair %d: max |E - oracle| = %.3e (bar %.3e)" % (mode, b, err, tol))
        assert err <= tol
        assert (got["E"][b][ref["E"][r] > 1e-36] > 0).all()


def test_config4_full_size_sampled_pairs():
    import torch

    wl = workloads.pair_workload("c4_b32_l8192")
    say("config 4 fused: GPU")
    xd, yd = to_dev(wl.x), to_dev(wl.y)
    value, desc, ws = pkg.sdtw_forward(xd, yd, wl.gamma, pkg.FUSED)
    dx, dy, E = pkg.sdtw_backward(desc, xd, yd, ws, want_E=True)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    got = {"value": value.cpu().numpy().astype(np.float64), "dx": dx.cpu().numpy().astype(np.float64),
           "dy": dy.cpu().numpy().astype(np.float64)}
    assert np.all(np.isfinite(got["value"])) and np.all(np.isfinite(got["dx"])) and np.all(np.isfinite(got["dy"]))
    # E summed over a row is at least 1 and dx_i = 2 sum_j E_ij (x_i - y_j): translation invariance
    tot = got["dx"].sum(axis=1) + got["dy"].sum(axis=1)
    assert np.abs(tot).max() <= 2e-2 * np.abs(got["dx"]).max()
    pairs = [3, 28]
    E3 = E[pairs[0]].cpu().numpy()
    # the same backward without the E output (the gradients are then formed where E is produced)
    dx2, dy2, _ = pkg.sdtw_backward(desc, xd, yd, ws)
    torch.cuda.synchronize()
    for a, b2 in ((dx, dx2), (dy, dy2)):
        assert (a - b2).abs().max().item() <= 1e-4 * a.abs().max().item()
    del ws, E, dx2, dy2
    torch.cuda.empty_cache()
    say("config 4 fused: oracle on pairs %s" % pairs)
    ref = oracle.batch(wl.x[pairs], wl.y[pairs], wl.gamma, nthreads=2, want_E=True)
    check_against({k: v for k, v in ref.items() if k != "E"}, got, pairs=pairs, what="c4")
    # pair 3's whole alignment matrix: 96 % of the macro-steps of this configuration are skipped as
    # provably zero, so a wrongly skipped one would show here
    tol = e_tolerance(wl.x[pairs[:1]], wl.y[pairs[:1]], wl.gamma)
    err = np.abs(E3 - ref["E"][0]).max()
    say("  c4 pair %d: max |E - oracle| = %.3e (bar %.3e)" % (pairs[0], err, tol))
    assert err <= tol
    assert (E3[ref["E"][0] > 1e-36] > 0).all()
    assert abs(E3.sum() - ref["E"][0].sum()) <= 1e-3 * ref["E"][0].sum()


# ------------------------------------------------------------------------------- barycenter
def teacher_forced_step(bw, mode, z, X, m, v, step, ws, consts, min_memory=False):
    """One library step on (z, m, v) and the oracle's step from the same state; returns the workspace."""
    import torch

    lr, b1, b2, eps = consts
    z_in = z.cpu().numpy().astype(np.float64)
    m_o, v_o = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)
    loss, dz, ws = pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, lr, b1, b2, eps, mode, workspace=ws, want_dz=True,
                                            min_memory=min_memory)
    torch.cuda.synchronize()
    z_o = z_in.copy()
    lo, dzo = oracle.barycenter_step(z_o, bw.X, bw.gamma, lr, b1, b2, eps, step, m_o, v_o)
    assert abs(loss.item() - lo) <= VALUE_RTOL * max(abs(lo), 1.0), "step %d loss %r vs %r" % (step, loss.item(), lo)
    g = dz.cpu().numpy().astype(np.float64)
    err = np.abs(g - dzo).max() / np.abs(dzo).max()
    say("  step %d: loss %.6g, max|dz| %.4g, rel err dz %.3e" % (step, lo, np.abs(dzo).max(), err))
    assert err <= GRAD_RTOL, "step %d dz rel err %.3e" % (step, err)
    # Adam's moments after the step, from the same moments before it
    mm, vv = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)
    assert np.abs(mm - m_o).max() <= GRAD_RTOL * np.abs(m_o).max(), "step %d m" % step
    assert np.abs(vv - v_o).max() <= 2 * GRAD_RTOL * np.abs(v_o).max(), "step %d v" % step
    # the update itself, given the library's own moments (Adam divides by |g| where g ~ 0,
    # so the comparison through the oracle's gradient would amplify rounding there)
    expect = z_in - lr * (mm / (1 - b1 ** step)) / (np.sqrt(vv / (1 - b2 ** step)) + eps)
    np.testing.assert_allclose(z.cpu().numpy(), expect, rtol=1e-5, atol=1e-6)
    return ws


@pytest.mark.parametrize("min_memory", [False, True])
@pytest.mark.parametrize("mode", ["unfused", "fused"])
def test_barycenter_steps_teacher_forced(mode, min_memory):
    import torch

    bw = workloads.barycenter_workload(K=8, L=96, D=6, seed=5)
    say("barycenter %s min_memory=%s" % (mode, min_memory))
    consts = (0.05, 0.9, 0.999, 1e-8)
    z = to_dev(bw.z0.copy())
    X = to_dev(bw.X)
    m = torch.zeros_like(z)
    v = torch.zeros_like(z)
    ws = None
    for step in (1, 2, 3):
        ws = teacher_forced_step(bw, MODES[mode], z, X, m, v, step, ws, consts, min_memory=min_memory)


def test_config5_barycenter_teacher_forced_and_trajectory():
    # K = 64, L = 512, D = 32, gamma = 1, fused, 50 Adam steps.  The library runs freely; at steps 1, 10,
    # 25 and 50 the oracle takes the same step from the library's state (z, m, v) and loss, gradient and
    # both moments are compared.  Late steps have z close to the sequences, where the norm expansion of
    # the cost cancels most.  The oracle also runs the 50 steps on its own: the two trajectories are
    # compared loosely at the end (Adam divides by sqrt(v), which amplifies rounding where dz ~ 0).
    import torch

    bw = workloads.barycenter_workload()
    say("config 5: K=%d L=%d D=%d gamma=%g, %d steps" % (bw.K, bw.L, bw.D, bw.gamma, bw.steps))
    consts = (bw.lr, 0.9, 0.999, 1e-8)
    z = to_dev(bw.z0.copy())
    X = to_dev(bw.X)
    m = torch.zeros_like(z)
    v = torch.zeros_like(z)
    ws = None
    z_o = bw.z0.astype(np.float64)
    m_o, v_o = np.zeros_like(z_o), np.zeros_like(z_o)
    losses, losses_o = [], []
    for step in range(1, bw.steps + 1):
        lo, _ = oracle.barycenter_step(z_o, bw.X, bw.gamma, consts[0], consts[1], consts[2], consts[3], step, m_o, v_o)
        losses_o.append(lo)
        if step in (1, 10, 25, 50):
            ws = teacher_forced_step(bw, pkg.FUSED, z, X, m, v, step, ws, consts)
            losses.append(None)
        else:
            loss, _, ws = pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, *consts, mode=pkg.FUSED, workspace=ws)
            losses.append(loss)
    torch.cuda.synchronize()
    assert binding.workspace_status(ws) == 0
    got = [None if l is None else l.item() for l in losses]
    assert got[-2] < got[1]
    # free-running trajectories: final point and the loss along the way
    zz = z.cpu().numpy().astype(np.float64)
    dev = np.abs(zz - z_o).max() / np.abs(z_o).max()
    say("  after %d free steps: max |z - oracle z| / max |z| = %.3e" % (bw.steps, dev))
    assert dev <= 1e-2
    for step in (2, 9, 24, 49):
        assert abs(got[step - 1] - losses_o[step - 1]) <= 1e-3 * max(abs(losses_o[step - 1]), 1.0), step
