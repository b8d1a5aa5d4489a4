"""Learned Butterfly extension through the C ABI against the float64 oracle: every supported length, both half
dtypes, blocks that are the DFT (where the result must be the plain convolution) and blocks moved away from it,
gradients of rows, spectrum and blocks, optional outputs, error codes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_06646_amd as lc
import workloads as wl
from gpu_harness import TOL, _compare, to_dev, to_f64
from oracle import lbfly

pytestmark = pytest.mark.gpu


def _inputs(B, H, N, io, seed=0, eps=0.1):
    """Rows and output gradients of unit variance, a decaying filter, and blocks that are the DFT moved by a complex
    perturbation of relative size eps (eps = 0: the fixed transform)."""
    r_u, r_k, r_D, r_dy, r_A = np.random.default_rng(88000 + 7 * N + seed).spawn(5)
    u_s, u_v = wl.quantize(r_u.standard_normal((B, H, N), dtype=np.float32), io)
    dy_s, dy_v = wl.quantize(r_dy.standard_normal((B, H, N), dtype=np.float32), io)
    t = np.arange(N, dtype=np.float64)[None, :]
    k = (r_k.standard_normal((H, N)) / np.sqrt(N) * np.exp(-4.0 * t / N)).astype(np.float32)
    D = r_D.standard_normal(H).astype(np.float32)
    Af, Ai = lbfly.dft_blocks(H, 2 * N)
    if eps:
        rl = 2 * N // 256
        mask = np.zeros(Af.shape)
        mask[:, :2] = 1.0
        mask[:, 2, :rl, :rl] = 1.0
        Af = Af + eps * mask * (r_A.standard_normal(Af.shape) + 1j * r_A.standard_normal(Af.shape))
        Ai = Ai + eps * mask * (r_A.standard_normal(Af.shape) + 1j * r_A.standard_normal(Af.shape))
    # the library takes the blocks as float32 (re, im): the oracle gets exactly those values
    Af32 = np.stack([Af.real, Af.imag], axis=-1).astype(np.float32)
    Ai32 = np.stack([Ai.real, Ai.imag], axis=-1).astype(np.float32)
    c = lambda a: a[..., 0].astype(np.float64) + 1j * a[..., 1].astype(np.float64)
    return u_s, u_v, dy_s, dy_v, k, D, Af32, Ai32, c(Af32), c(Ai32)


def _run(u_s, dy_s, k, D, Af32, Ai32, io, want=(True, True, True, True)):
    B, H, N = u_s.shape
    u, dy = to_dev(u_s, io), to_dev(dy_s, io)
    kd, Dd = torch.from_numpy(k).cuda(), torch.from_numpy(D).cuda()
    Af, Ai = torch.from_numpy(Af32).cuda(), torch.from_numpy(Ai32).cuda()
    shat = torch.full((H, 2 * N, 2), float("nan"), device="cuda")
    lc.longconv_lbfly_spectrum(kd, Dd, shat)
    y, du = torch.full_like(u, float("nan")), torch.full_like(u, float("nan"))
    dshat = torch.full_like(shat, float("nan"))
    dAf, dAi = torch.full_like(Af, float("nan")), torch.full_like(Ai, float("nan"))
    dk, dD = torch.full_like(kd, float("nan")), torch.full_like(Dd, float("nan"))
    ws = torch.empty(lc.longconv_lbfly_workspace_bytes(B, H, N, io), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    lc.longconv_lbfly_fwd(u, shat, Af, Ai, y)
    lc.longconv_lbfly_bwd(dy, u, shat, Af, Ai, du if want[0] else None, dshat if want[1] else None,
                          dAf if want[2] else None, dAi if want[3] else None, ws)
    if want[1]:
        lc.longconv_lbfly_spectrum_bwd(dshat, dk, dD)
    torch.cuda.synchronize()
    c = lambda t: t.cpu().numpy()[..., 0].astype(np.float64) + 1j * t.cpu().numpy()[..., 1].astype(np.float64)
    return dict(y=to_f64(y, io), du=to_f64(du, io), shat=c(shat), dshat=c(dshat), dAf=c(dAf), dAi=c(dAi),
                dk=dk.cpu().numpy().astype(np.float64), dD=dD.cpu().numpy().astype(np.float64))


def _ri(x):
    """complex [..., n] -> real [..., 2n] (re and im side by side), for the real-valued comparison helpers"""
    return np.concatenate([np.real(x), np.imag(x)], axis=-1)


def _check_blocks(got, want, N, tol, label):
    """The gradient of every stage's blocks over all heads to `tol`, and every single block (a sum with
    cancellation over as few as B * 16 columns, down to four entries for the last stage of N = 256: no averaging
    over entries) to 3 tol, relative to that block's own norm."""
    rl = 2 * N // 256
    worst = 0.0
    for s in range(3):
        r = 16 if s < 2 else rl
        e = wl.rel_l2(_ri(got[:, s, :r, :r]), _ri(want[:, s, :r, :r]))
        assert np.isfinite(e) and e <= tol, f"{label}: stage {s}: {e:.3e} > {tol:g}"
        for h in range(want.shape[0]):
            e = wl.rel_l2(_ri(got[h, s, :r, :r]), _ri(want[h, s, :r, :r]))
            worst = max(worst, e)
            assert np.isfinite(e) and e <= 3 * tol, f"{label}: head {h} stage {s}: {e:.3e} > {3 * tol:g}"
    outside = np.abs(got[:, 2]).copy()
    outside[:, :rl, :rl] = 0
    assert np.all(outside == 0), f"{label}: gradient outside the last stage's corner"
    return worst


CASES = [(256, wl.F16, 5, 3), (256, wl.BF16, 3, 520), (512, wl.BF16, 5, 3), (512, wl.F16, 1, 1), (1024, wl.F16, 7, 2),
         (1024, wl.BF16, 4, 3), (1024, wl.F16, 13, 1), (2048, wl.F16, 3, 2), (2048, wl.BF16, 5, 2)]


@pytest.mark.parametrize("N,io,B,H", CASES)
def test_learned_blocks_against_the_oracle(N, io, B, H):
    print(f"[lbfly] N={N} io={wl.DTYPE_NAMES[io]} B={B} H={H}", flush=True)
    u_s, u_v, dy_s, dy_v, k, D, Af32, Ai32, Af, Ai = _inputs(B, H, N, io)
    g = _run(u_s, dy_s, k, D, Af32, Ai32, io)
    shat = lbfly.spectrum(k, D)
    assert wl.rel_l2(_ri(g["shat"]), _ri(shat)) <= 1e-5
    ry = lbfly.lbfly_fwd(u_v, shat, Af, Ai)
    rdu, rdshat, rdAf, rdAi = lbfly.lbfly_bwd(dy_v, u_v, shat, Af, Ai)
    rdk, rdD = lbfly.spectrum_bwd(rdshat, N)
    tol = TOL[io]
    label = f"lbfly N={N} io={wl.DTYPE_NAMES[io]}"
    _compare({"y": g["y"], "du": g["du"], "dshat": _ri(g["dshat"]), "dk": g["dk"]},
             {"y": ry, "du": rdu, "dshat": _ri(rdshat), "dk": rdk}, tol, label)
    wf = _check_blocks(g["dAf"], rdAf, N, tol, label + " dAf")
    wi = _check_blocks(g["dAi"], rdAi, N, tol, label + " dAi")
    e_dD = float(np.max(np.abs(g["dD"] - rdD)) / max(np.sqrt(np.mean(rdD ** 2)), 1e-30))
    print(f"[lbfly] worst block dAf {wf:.2e} dAi {wi:.2e} dD {e_dD:.2e}", flush=True)
    assert e_dD <= tol


@pytest.mark.parametrize("N,io", [(256, wl.F16), (1024, wl.BF16), (2048, wl.F16)])
def test_dft_blocks_reproduce_the_plain_convolution(N, io):
    B, H = 3, 2
    u_s, u_v, dy_s, dy_v, k, D, Af32, Ai32, Af, Ai = _inputs(B, H, N, io, seed=1, eps=0.0)
    g = _run(u_s, dy_s, k, D, Af32, Ai32, io)
    k64, D64 = k.astype(np.float64), D.astype(np.float64)
    ry = oracle.longconv_fwd(u_v, k64, D64)
    rdu, rdk, rdD = oracle.longconv_bwd(dy_v, u_v, k64, D64)
    _compare({"y": g["y"], "du": g["du"], "dk": g["dk"]}, {"y": ry, "du": rdu, "dk": rdk}, TOL[io],
             f"lbfly with DFT blocks N={N} io={wl.DTYPE_NAMES[io]}")
    assert float(np.max(np.abs(g["dD"] - rdD)) / np.sqrt(np.mean(rdD ** 2))) <= TOL[io]


def test_full_size_of_the_timed_shape():
    """B=16, H=768, N=1024, bf16 rows: the shape `sweep --learned` times, in its launch configuration (rows of a head
    split over workgroups as there); every output of 24 heads (first, last, seeded ones) against the oracle."""
    N, io, B, H = 1024, wl.BF16, 16, 768
    u_s, u_v, dy_s, dy_v, k, D, Af32, Ai32, Af, Ai = _inputs(B, H, N, io, seed=3)
    g = _run(u_s, dy_s, k, D, Af32, Ai32, io)
    heads = sorted({0, H - 1, *np.random.default_rng(5).choice(H, size=22, replace=False).tolist()})
    shat = lbfly.spectrum(k[heads], D[heads])
    ry = lbfly.lbfly_fwd(u_v[:, heads], shat, Af[heads], Ai[heads])
    rdu, rdshat, rdAf, rdAi = lbfly.lbfly_bwd(dy_v[:, heads], u_v[:, heads], shat, Af[heads], Ai[heads])
    rdk, rdD = lbfly.spectrum_bwd(rdshat, N)
    tol = TOL[io]
    label = "lbfly full size"
    _compare({"y": g["y"][:, heads], "du": g["du"][:, heads], "dshat": _ri(g["dshat"][heads]), "dk": g["dk"][heads]},
             {"y": ry, "du": rdu, "dshat": _ri(rdshat), "dk": rdk}, tol, label)
    _check_blocks(g["dAf"][heads], rdAf, N, tol, label + " dAf")
    _check_blocks(g["dAi"][heads], rdAi, N, tol, label + " dAi")
    assert np.all(np.isfinite(g["y"])) and np.all(np.isfinite(g["dAf"])) and np.all(np.isfinite(g["dshat"]))


def test_optional_outputs_repeatability_and_error_codes():
    N, io, B, H = 512, wl.F16, 4, 3
    u_s, u_v, dy_s, dy_v, k, D, Af32, Ai32, Af, Ai = _inputs(B, H, N, io, seed=2)
    full = _run(u_s, dy_s, k, D, Af32, Ai32, io)
    again = _run(u_s, dy_s, k, D, Af32, Ai32, io)
    for name in ("y", "du", "dshat", "dAf", "dAi", "dk", "dD"):
        assert np.array_equal(full[name], again[name]), name          # fixed summation order
    only_du = _run(u_s, dy_s, k, D, Af32, Ai32, io, want=(True, False, False, False))
    assert np.array_equal(only_du["du"], full["du"]) and np.all(np.isnan(only_du["dshat"]))
    assert np.all(np.isnan(only_du["dAf"])) and np.all(np.isnan(only_du["dAi"]))
    no_du = _run(u_s, dy_s, k, D, Af32, Ai32, io, want=(False, True, True, True))
    assert np.all(np.isnan(no_du["du"])) and np.array_equal(no_du["dAf"], full["dAf"])
    assert np.array_equal(no_du["dshat"], full["dshat"])
    assert lc.longconv_lbfly_workspace_bytes(B, H, 4096, io) == 0            # longer than the on-chip buffers allow
    assert lc.longconv_lbfly_workspace_bytes(B, H, N, wl.F32) == 0           # half-precision rows only
    u32 = torch.zeros(B, H, N, device="cuda")
    shat = torch.zeros(H, 2 * N, 2, device="cuda")
    A = torch.from_numpy(Af32).cuda()
    with pytest.raises(lc.LongconvError, match="dtype"):
        lc.longconv_lbfly_fwd(u32, shat, A, A, torch.empty_like(u32))
    u = to_dev(u_s, io)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(lc.LongconvError, match="workspace"):
        lc.longconv_lbfly_bwd(u, u, shat, A, A, torch.empty_like(u), None, None, None, small)
