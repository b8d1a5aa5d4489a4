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


def check_full(inp: wl.Inputs, *, backward=True, label=""):
    """Whole-tensor parity of fwd (and bwd) against the oracle. Returns the error dict."""
    g = GpuRun(inp)
    tol = TOL[inp.w.dtype]
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    errs = {"y": wl.rel_l2(g.fwd(), oracle.longconv_fwd(inp.u, k64, D64))}
    if backward:
        du, dk, dD = g.bwd()
        rdu, rdk, rdD = oracle.longconv_bwd(inp.dy, inp.u, k64, D64)
        errs.update(du=wl.rel_l2(du, rdu), dk=wl.rel_l2(dk, rdk), dD=wl.rel_l2(dD, rdD))
    print(f"[parity] {label or inp.w.name} B{g.B} H{g.H} N{g.N}: " +
          " ".join(f"{k}={v:.2e}" for k, v in errs.items()) + f" (tol {tol:g})", flush=True)
    for name, e in errs.items():
        assert np.isfinite(e) and e <= tol, f"{name} rel-L2 {e:.3e} > {tol:g}"
    return errs


def check_sampled(inp: wl.Inputs, heads, *, backward=True, label=""):
    """Full-size GPU run checked on a sample: all batch rows of the heads in `heads`."""
    g = GpuRun(inp)
    tol = TOL[inp.w.dtype]
    hs = list(heads)
    k64, D64 = inp.k.astype(np.float64)[hs], inp.D.astype(np.float64)[hs]
    y = g.fwd()
    errs = {"y": wl.rel_l2(y[:, hs], oracle.longconv_fwd(inp.u[:, hs], k64, D64))}
    if backward:
        du, dk, dD = g.bwd()
        rdu, rdk, rdD = oracle.longconv_bwd(inp.dy[:, hs], inp.u[:, hs], k64, D64)
        errs.update(du=wl.rel_l2(du[:, hs], rdu), dk=wl.rel_l2(dk[hs], rdk), dD=wl.rel_l2(dD[hs], rdD))
        assert np.all(np.isfinite(du)) and np.all(np.isfinite(dk)) and np.all(np.isfinite(dD))
    assert np.all(np.isfinite(y))
    print(f"[parity/sampled heads={hs}] {label or inp.w.name}: " +
          " ".join(f"{k}={v:.2e}" for k, v in errs.items()) + f" (tol {tol:g})", flush=True)
    for name, e in errs.items():
        assert np.isfinite(e) and e <= tol, f"{name} rel-L2 {e:.3e} > {tol:g}"
    return errs
