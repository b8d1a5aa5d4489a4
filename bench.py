#!/usr/bin/env python3
"""Benchmark of the long-convolution hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic input, as a training
step would run it (the kernel changes every step, so its spectrum is recomputed):

    kernel-spectrum precompute  ->  forward  ->  backward (du, dk, dD in one call)

Inputs are resident in HBM before the timed region.  Each step uses the next of several
distinct buffer sets (more than the 256 MB last-level cache in total) so that reads come from
HBM rather than from cache.  The timed region is exactly K steps between two events on the launch
stream; the per-call durations (`segments_ms`, `roofline`) come from a second run of the same K
steps with an event between the three calls (each event costs a few microseconds of GPU time, so
it stays out of the timed region).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2|3|4a|...] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
CACHE_BYTES = 256 << 20        # last-level (Infinity) cache
# HBM bytes per launch group measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a copy kernel
# of known size: FETCH_SIZE x 2.0 KiB, WRITE_SIZE x 1.0 KiB), summed over the kernels of the group; see
# profiles/.
KIB = 1024
MEASURED_TRAFFIC = {
    # (backward: one kernel for du, dk and dD)
    "cfg2_B16_H768_N1024_bf16": {"fwd": (15883.1 * 2 + 24576.0) * KIB, "bwd": (28186.2 * 2 + 27672.0) * KIB},
    # (the convolution kernels read rows in 64-byte requests, which FETCH_SIZE x 2 over-counts: upper bound;
    # backward: the dk kernel, then the convolution kernel with the conjugate spectrum)
    "cfg3_B8_H256_N16384_fp16": {"fwd": (98875.7 * 2 + 65536.0) * KIB,
                                 "bwd": ((141672.5 + 98870.0) * 2 + 35911.8 + 65536.0) * KIB},
    # (inner convolution with pass A inside + pass C; backward: dk rows kernel + pass C + dD reduction, then
    # the convolution with the conjugate spectrum + pass C)
    "cfg4_B1_H128_N65536_fp16": {"fwd": ((49954.9 + 33050.9) * 2 + 65577.8 + 16384.0) * KIB,
                                 "bwd": ((18854.9 + 32938.6 + 3.2 + 49963.5 + 33050.9) * 2 + 77826.8 + 32768.0 + 0.5 +
                                         65563.6 + 16384.0) * KIB},
}

def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Sets:
    """Device buffers for one workload: `nsets` rotating copies of the big tensors."""

    def __init__(self, w: wl.Workload, lc, torch, min_total=2 * CACHE_BYTES + (64 << 20)):
        self.w = w
        td = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[w.dtype]
        per_set = 4 * w.B * w.H * w.N * wl.DTYPE_BYTES[w.dtype]
        self.nsets = max(2, int(np.ceil(min_total / per_set)))
        g = torch.Generator(device="cuda").manual_seed(20230213 * 10 + w.wid)
        shape = (w.B, w.H, w.N)
        self.u = [torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(td) for _ in range(self.nsets)]
        self.dy = [torch.randn(shape, generator=g, device="cuda", dtype=torch.float32).to(td) for _ in range(self.nsets)]
        self.y = [torch.empty(shape, device="cuda", dtype=td) for _ in range(self.nsets)]
        self.du = [torch.empty(shape, device="cuda", dtype=td) for _ in range(self.nsets)]
        # kernel and skip term: the seeded host generator (distribution matters for nothing but realism)
        inp = wl.generate(w, B=1)
        self.k = torch.from_numpy(inp.k).cuda()
        self.D = torch.from_numpy(inp.D).cuda()
        self.dk = torch.empty_like(self.k)
        self.dD = torch.empty_like(self.D)
        self.kspec = lc.new_kspec(w.H, w.N, w.dtype)
        self.ws = lc.new_workspace(w.B, w.H, w.N, w.dtype, True)


def run_workload(key, steps, warmup, lc, torch):
    w = wl.WORKLOADS[key]
    S = Sets(w, lc, torch)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = [[ev() for _ in range(4)] for _ in range(steps)]

    def step(i, m=None):
        j = i % S.nsets
        if m: m[0].record()
        lc.longconv_kspec_compute(S.k, S.D, S.kspec, w.dtype, S.ws)
        if m: m[1].record()
        lc.longconv_fwd(S.u[j], S.k, S.D, S.y[j], S.ws, kspec=S.kspec)
        if m: m[2].record()
        lc.longconv_bwd(S.dy[j], S.u[j], S.k, S.D, S.du[j], S.dk, S.dD, S.ws, kspec=S.kspec)
        if m: m[3].record()

    for i in range(warmup):
        step(i)
    # timed region: exactly `steps` steps between two events on the launch stream, nothing in between
    e0, e1 = ev(), ev()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    step_ms = e0.elapsed_time(e1) / steps
    # instrumented region: the same steps again with an event between the three calls (each event costs a few
    # microseconds of GPU time, which is why it is kept out of the timed region); gives the per-launch durations
    for i in range(steps):
        step(warmup + steps + i, marks[i])
    torch.cuda.synchronize()
    seg = np.array([[m[a].elapsed_time(m[a + 1]) for a in range(3)] for m in marks])   # ms
    seg_avg = seg.mean(axis=0)
    fwd_b, bwd_b = wl.algorithmic_bytes(w.B, w.H, w.N, w.dtype)
    # algorithmic bytes of each call (the spectrum's read of k is already in fwd's figure)
    seg_bytes = {"kspec": 0, "fwd": fwd_b, "bwd": bwd_b}
    names = list(seg_bytes)
    res = {
        "workload": w.name, "B": w.B, "H": w.H, "N": w.N, "io": wl.DTYPE_NAMES[w.dtype],
        "plan": lc.longconv_plan_string(w.N, w.dtype), "buffer_sets": S.nsets,
        "ms_per_step": float(step_ms), "wall_ms_per_step": wall_ms, "ms_per_step_instrumented": float(seg_avg.sum()),
        "bytes_per_step": fwd_b + bwd_b,
        "GBps": (fwd_b + bwd_b) / (step_ms * 1e-3) / 1e9,
        "segments": {n: {"ms": float(seg_avg[i]), "ms_min": float(seg[:, i].min()),
                         "GBps": (seg_bytes[n] / (seg_avg[i] * 1e-3) / 1e9) if seg_bytes[n] else None}
                     for i, n in enumerate(names)},
    }
    ff, bf = wl.algorithmic_flops(w.B, w.H, w.N)
    res["TFLOPs_algorithmic"] = (ff + bf) / (step_ms * 1e-3) / 1e12
    res["frac_hbm"] = res["GBps"] / HBM_PEAK_GBS
    del S
    torch.cuda.empty_cache()
    return res, seg_bytes


def cpu_baseline(key):
    """The float64 oracle, as it stands, on the host cores: whole workload if it is a few seconds of
    work, otherwise all batch rows of a subset of heads (cost is linear in heads)."""
    import oracle
    w = wl.WORKLOADS[key]
    macs_per_head = 3 * w.B * w.N * w.N / 2          # fwd + du + dk
    budget = 15.0 * 10e9                             # about 15 s at ~10 GMAC/s
    heads = int(max(1, min(w.H, budget // macs_per_head)))
    inp = wl.generate(w, H=heads)
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    t0 = time.perf_counter()
    oracle.longconv_fwd(inp.u, k64, D64)
    oracle.longconv_bwd(inp.dy, inp.u, k64, D64)
    dt = time.perf_counter() - t0
    fwd_b, bwd_b = wl.algorithmic_bytes(w.B, heads, w.N, w.dtype)
    return {"value": (fwd_b + bwd_b) / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{heads} of {w.H} heads, all {w.B} batch rows, fwd+bwd, {dt:.2f} s "
                      f"(float64 direct O(N^2) sums; scales linearly in heads)",
            "ms_per_step_scaled": dt * 1e3 * w.H / heads}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="2", choices=list(wl.WORKLOADS))
    ap.add_argument("--also", default="3,4a", help="comma list of further workloads reported under 'targets'")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 64 MiB device copies (reference for scaling rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    import paper_2302_06646_amd as lc
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    lc.longconv_init()
    if a.copy_probe:
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    res, seg_bytes = run_workload(a.workload, a.steps, a.warmup, lc, torch)
    log(json.dumps(res, indent=1))
    # dominant kernel = the launch group with the largest share of the step
    dom = max(("fwd", "bwd"), key=lambda n: res["segments"][n]["ms"])
    dom_gbps = res["segments"][dom]["GBps"]
    out = {
        "metric": "long-conv fwd+bwd ms, effective GB/s and % HBM roofline at BxHxN",
        "value": res["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": res["workload"], "B": res["B"], "H": res["H"], "N": res["N"], "io": res["io"],
                   "step": "kspec+fwd+bwd(du,dk,dD)", "plan": res["plan"], "buffer_sets": res["buffer_sets"]},
        "pct_hbm_roofline": 100.0 * res["frac_hbm"],
        "TFLOPs_algorithmic": res["TFLOPs_algorithmic"],
        "segments_ms": {n: v["ms"] for n, v in res["segments"].items()},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": dom_gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": dom_gbps / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC.get(res["workload"], {}).get(dom),
                     "algorithmic_bytes_per_launch": seg_bytes[dom]},
    }
    targets = []
    for key in [k for k in a.also.split(",") if k and k != a.workload]:
        r, _ = run_workload(key, max(10, a.steps // 2), max(3, a.warmup // 2), lc, torch)
        log(json.dumps(r, indent=1))
        targets.append({"workload": r["workload"], "ms_per_step": r["ms_per_step"], "GBps": r["GBps"],
                        "pct_hbm_roofline": 100 * r["frac_hbm"],
                        "fwd_ms": r["segments"]["fwd"]["ms"],
                        "fwd_pct_hbm_roofline": 100 * r["segments"]["fwd"]["GBps"] / HBM_PEAK_GBS})
    out["targets"] = targets
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(a.workload)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
