"""Helpers for the GPU parity tests: upload seeded inputs, call the library through its
C-ABI binding, download results, compare with the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2302_06646_amd as lc
import workloads as wl

TOL = {wl.F32: 1e-5, wl.F16: 3e-3, wl.BF16: 3e-3}     # relative L2 bounds per I/O dtype
_TD = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}


def to_dev(store: np.ndarray, dtype: int) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(store))
    if dtype == wl.BF16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_f64(t: torch.Tensor, dtype: int) -> np.ndarray:
    t = t.cpu()
    if dtype == wl.BF16:
        return wl.storage_to_f64(t.view(torch.uint16).numpy(), dtype)
    return t.numpy().astype(np.float64)


class GpuRun:
    """Device copies of one input set plus output buffers and workspace."""

    def __init__(self, inp: wl.Inputs):
        self.inp = inp
        w = inp.w
        self.io = w.dtype
        self.B, self.H, self.N = inp.u_store.shape
        self.u = to_dev(inp.u_store, w.dtype)
        self.dy = to_dev(inp.dy_store, w.dtype)
        self.k = torch.from_numpy(inp.k).cuda()
        self.D = torch.from_numpy(inp.D).cuda()
        self.y = torch.full_like(self.u, float("nan"))
        self.du = torch.full_like(self.u, float("nan"))
        self.dk = torch.full_like(self.k, float("nan"))
        self.dD = torch.full_like(self.D, float("nan"))
        self.ws = lc.new_workspace(self.B, self.H, self.N, self.io, True)

    def fwd(self, kspec=None):
        lc.longconv_fwd(self.u, self.k, self.D, self.y, self.ws, kspec=kspec)
        torch.cuda.synchronize()
        return to_f64(self.y, self.io)

    def bwd(self, kspec=None, du=True, dk=True, dD=True):
        lc.longconv_bwd(self.dy, self.u, self.k, self.D, self.du if du else None, self.dk if dk else None,
                        self.dD if dD else None, self.ws, kspec=kspec)
        torch.cuda.synchronize()
        return (to_f64(self.du, self.io), self.dk.cpu().numpy().astype(np.float64),
                self.dD.cpu().numpy().astype(np.float64))

    def kspec(self):
        ks = lc.new_kspec(self.H, self.N, self.io)
        lc.longconv_kspec_compute(self.k, self.D, ks, self.io, self.ws)
        return ks


DD_TOL = 1e-5      # dD is a plain fp32 dot product of the (already quantised) rows on every path


def _row_errs(x, ref):
    """Relative L2 error of every row (last axis) of x against ref; rows whose reference is zero count their
    absolute error."""
    x = np.asarray(x, dtype=np.float64).reshape(-1, x.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    num = np.linalg.norm(x - ref, axis=1)
    den = np.linalg.norm(ref, axis=1)
    return np.where(den > 0, num / np.where(den > 0, den, 1.0), num)


def _compare(got: dict, want: dict, tol: float, label: str, dd_tol: float = None):
    """Whole-tensor relative L2 of every output, and the worst single row (y, du: one (b,h) sequence; dk: one
    head) so that one wrong row cannot hide in the norm of thousands of good ones.  dD: whole vector against
    DD_TOL, and every head against DD_TOL of the size a head's dD typically has (||u_h|| ||dy_h|| / sqrt(B N) up
    to a constant: the rms of the vector stands in for it)."""
    dd_tol = DD_TOL if dd_tol is None else dd_tol
    errs, worst = {}, {}
    for name in got:
        errs[name] = wl.rel_l2(got[name], want[name])
        if name == "dD":
            scale = max(float(np.sqrt(np.mean(np.square(want[name])))), 1e-30)
            worst[name] = float(np.max(np.abs(got[name] - want[name])) / scale)
        else:
            worst[name] = float(np.max(_row_errs(got[name], want[name])))
    print(f"[parity] {label}: " + " ".join(f"{k}={v:.2e}(row {worst[k]:.2e})" for k, v in errs.items()) +
          f" (tol {tol:g}, dD {dd_tol:g})", flush=True)
    for name, e in errs.items():
        t = dd_tol if name == "dD" else tol
        assert np.isfinite(e) and e <= t, f"{label}: {name} rel-L2 {e:.3e} > {t:g}"
        assert np.isfinite(worst[name]) and worst[name] <= t, f"{label}: worst row of {name} {worst[name]:.3e} > {t:g}"
    return errs


def check_full(inp: wl.Inputs, *, backward=True, label="", dd_tol=None):
    """Whole-tensor and per-row parity of fwd (and bwd) against the oracle. Returns the error dict."""
    g = GpuRun(inp)
    tol = TOL[inp.w.dtype]
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    got = {"y": g.fwd()}
    want = {"y": oracle.longconv_fwd(inp.u, k64, D64)}
    if backward:
        du, dk, dD = g.bwd()
        rdu, rdk, rdD = oracle.longconv_bwd(inp.dy, inp.u, k64, D64)
        got.update(du=du, dk=dk, dD=dD)
        want.update(du=rdu, dk=rdk, dD=rdD)
    return _compare(got, want, tol, f"{label or inp.w.name} B{g.B} H{g.H} N{g.N}", dd_tol)


def sample_heads(H: int, B: int, seed: int, min_rows: int = 32):
    """First and last head plus seeded ones in between, enough for at least `min_rows` (b,h) rows."""
    n = max(2, -(-min_rows // B))
    n = min(n, H)
    hs = {0, H - 1}
    rng = np.random.default_rng(seed)
    while len(hs) < n:
        hs.add(int(rng.integers(0, H)))
    return sorted(hs)


def check_sampled(inp: wl.Inputs, heads, *, backward=True, label=""):
    """Full-size GPU run checked on a sample: all batch rows of the heads in `heads`, per row and as a whole;
    everything outside the sample must at least be finite."""
    g = GpuRun(inp)
    tol = TOL[inp.w.dtype]
    hs = list(heads)
    k64, D64 = inp.k.astype(np.float64)[hs], inp.D.astype(np.float64)[hs]
    y = g.fwd()
    assert np.all(np.isfinite(y))
    got = {"y": y[:, hs]}
    want = {"y": oracle.longconv_fwd(inp.u[:, hs], k64, D64)}
    if backward:
        du, dk, dD = g.bwd()
        assert np.all(np.isfinite(du)) and np.all(np.isfinite(dk)) and np.all(np.isfinite(dD))
        rdu, rdk, rdD = oracle.longconv_bwd(inp.dy[:, hs], inp.u[:, hs], k64, D64)
        got.update(du=du[:, hs], dk=dk[hs], dD=dD[hs])
        want.update(du=rdu, dk=rdk, dD=rdD)
    return _compare(got, want, tol, f"{label or inp.w.name} sampled heads {hs if len(hs) <= 8 else str(len(hs)) + ' heads'}")
