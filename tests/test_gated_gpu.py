"""Gated long convolution (output times a second sequence) and its backward through the C ABI against the float64
oracle: every plan family, all three I/O dtypes, optional outputs."""
import numpy as np
import pytest
import torch

import paper_2302_06646_amd as lc
import workloads as wl
from gpu_harness import TOL, DD_TOL, _compare, to_dev, to_f64
from oracle import gated

pytestmark = pytest.mark.gpu


def _inputs(N, io, B, H, seed=0):
    kind = {wl.F32: "decay256", wl.F16: "decay_alpha_squash", wl.BF16: "squash_pool"}[io]
    w = wl.Workload(6, B, H, N, io, kind)
    inp = wl.generate(w, seed_extra=seed)
    g32 = np.random.default_rng(991 + N + seed).standard_normal((B, H, N), dtype=np.float32)
    g_s, g_v = wl.quantize(g32, io)
    return inp, g_s, g_v


def _run(inp, g_s, want_du=True, want_dk=True, want_dD=True, want_dg=True):
    io = inp.w.dtype
    B, H, N = inp.u_store.shape
    u, dy, g = to_dev(inp.u_store, io), to_dev(inp.dy_store, io), to_dev(g_s, io)
    k, D = torch.from_numpy(inp.k).cuda(), torch.from_numpy(inp.D).cuda()
    y = torch.full_like(u, float("nan"))
    du, dg = torch.full_like(u, float("nan")), torch.full_like(u, float("nan"))
    dk, dD = torch.full_like(k, float("nan")), torch.full_like(D, float("nan"))
    ws = lc.new_workspace(B, H, N, io, 2)
    lc.longconv_fwd_gated(u, k, D, g, y, ws)
    lc.longconv_bwd_gated(dy, g, u, k, D, du if want_du else None, dk if want_dk else None,
                          dD if want_dD else None, dg if want_dg else None, ws)
    torch.cuda.synchronize()
    return (to_f64(y, io), to_f64(du, io), dk.cpu().numpy().astype(np.float64), dD.cpu().numpy().astype(np.float64),
            to_f64(dg, io))


CASES = [(1024, wl.F32), (256, wl.BF16), (1024, wl.BF16), (2048, wl.F16), (4096, wl.BF16), (16384, wl.F16),
         (65536, wl.F16)]


@pytest.mark.parametrize("N,io", CASES)
def test_gated_layer_against_the_oracle(N, io):
    B, H = (3, 2) if N <= 16384 else (1, 2)
    inp, g_s, g_v = _inputs(N, io, B, H)
    y, du, dk, dD, dg = _run(inp, g_s)
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    ry = gated.gated_fwd(inp.u, k64, D64, g_v)
    rdu, rdk, rdD, rdg = gated.gated_bwd(inp.dy, g_v, inp.u, k64, D64)
    tol = TOL[io]
    errs = _compare({"y": y, "du": du, "dk": dk, "dg": dg}, {"y": ry, "du": rdu, "dk": rdk, "dg": rdg}, tol,
                    f"gated N={N} io={wl.DTYPE_NAMES[io]}")
    e_dD = wl.rel_l2(dD, rdD)
    assert e_dD <= DD_TOL, e_dD        # the fp32 sum of dy g u from the three tensors, on every dtype
    assert errs


def test_optional_outputs_and_error_codes():
    inp, g_s, g_v = _inputs(1024, wl.BF16, 2, 2)
    y, du, dk, dD, dg = _run(inp, g_s, want_du=False, want_dk=False, want_dD=False)
    assert np.all(np.isnan(du)) and np.all(np.isnan(dk)) and np.all(np.isnan(dD))
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    rdg = gated.gated_bwd(inp.dy, g_v, inp.u, k64, D64)[3]
    assert wl.rel_l2(dg, rdg) <= TOL[wl.BF16]
    y2, du2, dk2, dD2, dg2 = _run(inp, g_s, want_dg=False)
    assert np.all(np.isnan(dg2)) and np.all(np.isfinite(du2))
    # a backward workspace without room for dz is refused before anything is launched
    io = wl.BF16
    B, H, N = inp.u_store.shape
    u, dy, g = to_dev(inp.u_store, io), to_dev(inp.dy_store, io), to_dev(g_s, io)
    k, D = torch.from_numpy(inp.k).cuda(), torch.from_numpy(inp.D).cuda()
    small = lc.new_workspace(B, H, N, io, 1)
    with pytest.raises(lc.LongconvError, match="workspace"):
        lc.longconv_bwd_gated(dy, g, u, k, D, torch.empty_like(u), None, None, None, small)
    assert lc.longconv_workspace_bytes(B, H, N, io, 2) >= lc.longconv_workspace_bytes(B, H, N, io, 1) + B * H * N * 2
