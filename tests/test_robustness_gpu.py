"""Further GPU cases through the C-ABI binding: every length with both half dtypes and an odd batch,
kernels of extreme magnitude, launches on a side stream and under HIP graph capture."""
from __future__ import annotations

import dataclasses

import numpy as np
import pytest

import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _need_gpu_and_default_options():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2302_06646_amd as lc
    for name, value in lc.OPTION_DEFAULTS.items():      # whatever the environment or an earlier test left
        lc.longconv_set_option(name, value)
    yield
    for name, value in lc.OPTION_DEFAULTS.items():
        lc.longconv_set_option(name, value)


def _opt(name, value):
    import paper_2302_06646_amd as lc
    lc.longconv_set_option(name, value)


def _w(key, **kw):
    return dataclasses.replace(wl.WORKLOADS[key], **kw)


@pytest.mark.parametrize("io", [wl.F16, wl.BF16])
@pytest.mark.parametrize("N", [256, 512, 1024, 2048, 4096, 8192, 16384])
def test_every_single_pass_length_half_io_odd_batch(N, io):
    # one case per kernel family and tile count; B = 3 leaves the last row pair half empty; two heads only, so
    # that dD (one number per head, a sum of B N products of random sign that can come out small) is held to
    # its definition: the fp32 dot product of the raw rows, not a by-product of the rounded transforms
    from gpu_harness import check_full
    check_full(wl.generate(_w("2", N=N, dtype=io), B=3, H=2), label=f"N={N} io={wl.DTYPE_NAMES[io]}")


@pytest.mark.parametrize("io", [wl.F16, wl.BF16])
def test_longest_sequence_half_io(io):
    from gpu_harness import check_full
    check_full(wl.generate(_w("4b", dtype=io), B=2, H=1), label=f"N=131072 io={wl.DTYPE_NAMES[io]}")


@pytest.mark.parametrize("key,B,H", [("2", 4, 4), ("3", 2, 4), ("4a", 2, 4)])
def test_kernel_magnitudes_per_head(key, B, H):
    """Heads of different magnitude in one call, checked head by head (a whole-tensor norm would hide a
    small head behind a large one), and an all-zero head with D = 0, which must give exact zeros.  (Heads
    much further from one: tests/test_dynamic_range_gpu.py.)"""
    from gpu_harness import GpuRun, TOL
    import oracle
    inp = wl.generate(wl.WORKLOADS[key], B=B, H=H)
    scale = np.array([1.0 / 64, 1.0, 64.0, 0.0], dtype=np.float32)[:H]
    k = (inp.k * scale[:, None]).astype(np.float32)
    D = (inp.D * scale).astype(np.float32)
    inp = dataclasses.replace(inp, k=k, D=D)
    g = GpuRun(inp)
    y = g.fwd()
    du, dk, dD = g.bwd()
    k64, D64 = k.astype(np.float64), D.astype(np.float64)
    ry = oracle.longconv_fwd(inp.u, k64, D64)
    rdu, rdk, rdD = oracle.longconv_bwd(inp.dy, inp.u, k64, D64)
    tol = TOL[inp.w.dtype]
    for h in range(H):
        if scale[h] == 0.0:
            assert np.all(y[:, h] == 0.0) and np.all(du[:, h] == 0.0)
        else:
            ey, edu = wl.rel_l2(y[:, h], ry[:, h]), wl.rel_l2(du[:, h], rdu[:, h])
            print(f"[magnitude] {inp.w.name} head {h} scale {scale[h]:g}: y={ey:.2e} du={edu:.2e}", flush=True)
            assert ey <= tol and edu <= tol
        assert wl.rel_l2(dk[h], rdk[h]) <= tol       # dk does not depend on k: same accuracy for every head
    assert wl.rel_l2(dD, rdD) <= 1e-5                # dD: fp32 dot product of the rows on every path


def test_side_stream_matches_default_stream():
    import paper_2302_06646_amd as lc
    from gpu_harness import GpuRun
    g = GpuRun(wl.generate(wl.WORKLOADS["2"], B=4, H=4))
    y0 = g.fwd().copy()
    du0, dk0, dD0 = [a.copy() for a in g.bwd()]
    for t in (g.y, g.du, g.dk, g.dD):
        t.zero_()
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):                      # the binding picks up torch's current stream
        lc.longconv_fwd(g.u, g.k, g.D, g.y, g.ws)
    lc.longconv_bwd(g.dy, g.u, g.k, g.D, g.du, g.dk, g.dD, g.ws, stream=st)      # and takes an explicit one
    st.synchronize()
    from gpu_harness import to_f64
    assert np.array_equal(to_f64(g.y, g.io), y0)
    assert np.array_equal(to_f64(g.du, g.io), du0)
    assert np.array_equal(g.dk.cpu().numpy().astype(np.float64), dk0)
    assert np.array_equal(g.dD.cpu().numpy().astype(np.float64), dD0)


@pytest.mark.parametrize("key,B,H", [("2", 4, 8), ("3", 2, 2), ("4a", 1, 2)])
def test_step_under_graph_capture_replays_bitwise(key, B, H):
    """The library allocates nothing and never synchronises, so a whole step (spectrum, forward, both
    backward calls) can be captured into a HIP graph.  Every replay, with eager work and
    synchronisations between replays, must reproduce the eager results bit for bit."""
    import paper_2302_06646_amd as lc
    from gpu_harness import GpuRun
    g = GpuRun(wl.generate(wl.WORKLOADS[key], B=B, H=H))
    ks = lc.new_kspec(g.H, g.N, g.io)

    def step():
        lc.longconv_kspec_compute(g.k, g.D, ks, g.io, g.ws)
        lc.longconv_fwd(g.u, g.k, g.D, g.y, g.ws, kspec=ks)
        lc.longconv_bwd(g.dy, g.u, g.k, g.D, None, g.dk, g.dD, g.ws, kspec=ks)
        lc.longconv_bwd(g.dy, g.u, g.k, g.D, g.du, None, None, g.ws, kspec=ks)

    outs = (g.y, g.du, g.dk, g.dD)
    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        step()                                      # warm-up on the capture stream (tables, attributes)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=st):
            step()
    torch.cuda.synchronize()
    for r in range(3):
        for t in outs:
            t.fill_(float("nan"))                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, want in zip(outs, ref):
            assert torch.equal(t.view(torch.uint8), want.view(torch.uint8)), f"replay {r} differs"


@pytest.mark.parametrize("N,B,H,io", [(16384, 6, 129, wl.F16), (4096, 5, 771, wl.BF16), (8192, 3, 300, wl.BF16)])
def test_persistent_workgroups_ragged_item_count(N, B, H, io):
    """More (head, pair) items than resident workgroups, not a multiple of them, odd batch: every item must be
    processed exactly once.  Sampled heads against the oracle, and every output element against the staged
    in-place kernel (a different code path with one workgroup per item)."""
    import paper_2302_06646_amd as lc
    from gpu_harness import GpuRun, TOL, check_sampled, to_f64
    inp = wl.generate(_w("3", N=N, dtype=io), B=B, H=H)
    check_sampled(inp, [0, H // 2, H - 1], label=f"ragged N={N} B={B} H={H}")
    g = GpuRun(inp)
    y = g.fwd().copy()
    du, dk, dD = [a.copy() for a in g.bwd()]
    _opt("staged_kernel", 1)
    g2 = GpuRun(inp)
    y2 = g2.fwd()
    du2, dk2, dD2 = g2.bwd()
    tol = 2 * TOL[io]
    for h0 in range(0, H, 16):                      # block-wise, so that one missing head cannot hide in the norm
        sl = slice(h0, min(H, h0 + 16))
        assert wl.rel_l2(y[:, sl], y2[:, sl]) <= tol and wl.rel_l2(du[:, sl], du2[:, sl]) <= tol, f"heads {sl}"
        assert wl.rel_l2(dk[sl], dk2[sl]) <= tol, f"dk heads {sl}"
    assert wl.rel_l2(dD, dD2) <= tol


@pytest.mark.parametrize("io", [wl.F16, wl.BF16])
@pytest.mark.parametrize("N", [65536, 131072])
def test_pass_a_inside_the_inner_kernel(N, io):
    """N = 65536, 131072 (outer radix 4, 8): the convolutions, the spectrum and (N = 65536) dk take pass A while
    staging their rows.  Odd batch (the last pair has one row), both half dtypes, against the oracle and against
    the separate pass A."""
    from gpu_harness import GpuRun, TOL, check_full
    inp = wl.generate(_w("4a", N=N, dtype=io), B=3, H=1 if N > 65536 else 2)
    check_full(inp, label=f"pass A fused, io={wl.DTYPE_NAMES[io]}")
    g = GpuRun(inp)
    y = g.fwd().copy()
    du, dk, dD = (a.copy() for a in g.bwd())
    _opt("fuse_pass_a", 0)
    g2 = GpuRun(inp)
    y2 = g2.fwd()
    du2, dk2, dD2 = g2.bwd()
    tol = 2 * TOL[io]
    assert wl.rel_l2(y, y2) <= tol and wl.rel_l2(du, du2) <= tol
    assert wl.rel_l2(dk, dk2) <= tol and wl.rel_l2(dD, dD2) <= tol
    assert not np.array_equal(y, y2)          # the two paths round differently: the switch did take effect
    if N == 65536:
        assert not np.array_equal(dk, dk2)    # dk: outer radix 8 from the rows against radix 4 from a workspace


@pytest.mark.parametrize("io", [wl.F16, wl.BF16])
@pytest.mark.parametrize("N,B,H", [(256, 5, 7), (512, 1, 5), (1024, 7, 9), (1024, 16, 3), (2048, 3, 6)])
def test_backward_in_one_kernel(N, B, H, io):
    """Single-pass plans up to 4096 points: a call that asks for du and dk/dD runs one kernel (one read of dy
    and u, one transform of dy).  Against the oracle, and against the separate du and dk kernels: du sees the
    same arithmetic in both (bitwise equal), dk sums the same products with the roles of the packed and the
    fp32 operand swapped."""
    from gpu_harness import GpuRun, TOL, check_full
    inp = wl.generate(_w("2", N=N, dtype=io), B=B, H=H)
    check_full(inp, label=f"fused backward, io={wl.DTYPE_NAMES[io]}")
    g = GpuRun(inp)
    du, dk, dD = (a.copy() for a in g.bwd())
    du_only = g.bwd(dk=False, dD=False)[0].copy()          # du alone: the convolution kernel
    _opt("fuse_bwd", 0)
    g2 = GpuRun(inp)
    du2, dk2, dD2 = g2.bwd()
    tol = 2 * TOL[io]
    assert np.array_equal(du_only, du2)
    assert wl.rel_l2(du, du2) <= tol and wl.rel_l2(dk, dk2) <= tol and wl.rel_l2(dD, dD2) <= tol
    assert not np.array_equal(dk, dk2)        # the switch did take effect


@pytest.mark.parametrize("N,B,H,io", [(4096, 128, 32, wl.F16), (1024, 37, 3, wl.BF16), (16384, 12, 5, wl.F16)])
def test_few_heads_batch_dealt_to_several_workgroups(N, B, H, io):
    """With few heads the pairs of a head are dealt to several workgroups of the dk kernels and the partial dk and
    dD summed in a fixed order: against the oracle (whole tensors; the first shape is the one of the paper's
    block-size table, B = 128, H = 32, N = 4096), and bitwise repeatable call to call."""
    from gpu_harness import GpuRun, check_full
    inp = wl.generate(_w("2", N=N, dtype=io), B=B, H=H)
    check_full(inp, label=f"few heads N={N} B={B} H={H}")
    g = GpuRun(inp)
    du0, dk0, dD0 = (a.copy() for a in g.bwd())
    for _ in range(3):
        g.dk.fill_(float("nan")); g.dD.fill_(float("nan"))
        du1, dk1, dD1 = g.bwd()
        assert np.array_equal(dk1, dk0) and np.array_equal(dD1, dD0) and np.array_equal(du1, du0)
    dk_only = g.bwd(du=False)[1].copy()              # partial request: the separate dk kernel, also dealt out
    assert wl.rel_l2(dk_only, dk0) <= 2 * 3e-3


@pytest.mark.parametrize("io", [wl.F16, wl.BF16])
@pytest.mark.parametrize("N", [32768, 65536, 131072])
def test_single_row_batch_uses_the_hermitian_symmetry_of_its_chunks(N, io):
    """B = 1 in the multi-pass split: the row is real, so chunk R - k1 of the outer split is the complex conjugate
    of chunk k1; the inner kernels compute the chunks up to R/2 only and pass C fills in the rest.  Against the
    oracle, and against the plan with the separate pass A, which computes every chunk."""
    from gpu_harness import GpuRun, TOL, check_full
    inp = wl.generate(_w("4a", N=N, dtype=io), B=1, H=3 if N < 131072 else 2)
    check_full(inp, label=f"single row N={N} io={wl.DTYPE_NAMES[io]}")
    g = GpuRun(inp)
    y = g.fwd().copy()
    du, dk, dD = (a.copy() for a in g.bwd())
    _opt("fuse_pass_a", 0)
    g2 = GpuRun(inp)
    y2 = g2.fwd()
    du2, dk2, dD2 = g2.bwd()
    tol = 2 * TOL[io]
    assert wl.rel_l2(y, y2) <= tol and wl.rel_l2(du, du2) <= tol and wl.rel_l2(dk, dk2) <= tol
