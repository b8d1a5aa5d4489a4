#!/usr/bin/env python3
"""Benchmark of the long-convolution hot path on one MI355X.

One "step" = one pass of the whole path over one batch of synthetic input, as a training
step runs it (the kernel changes every step, so its spectrum is recomputed: "cold spectrum"):

    kernel-spectrum precompute  ->  forward  ->  backward (du, dk, dD in one call)

Headline workload: B=8, H=256, N=16384, fp16 I/O (the N=16K target configuration); the N=64K
target (B=1, H=128) and the language-model-width block (B=16, H=768, N=1024, bf16) follow under
`targets`, each with its own roofline object.

Inputs are resident in HBM before the timed region.  Each step uses the next of several distinct
buffer sets (more than twice the 256 MB last-level cache in total) so that reads come from HBM
rather than from cache.  The timed region is exactly K steps between two events on the launch
stream.  Further regions, each again K steps between events on the same stream:
  * per-call durations: an event between the calls of a step (the backward call split into its
    dk/dD part and its du part where the plan runs them as separate kernels anyway), median and
    minimum over the K steps;
  * warm spectrum: forward + backward with the cached spectrum (inference-like / frozen kernel);
  * cache-hot: the same buffer set every step (labelled as such; never the headline).
A plain device copy is timed in the same run (copy bandwidth of the box).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3|4a|2|...] [--also 4a,2] [--no-cpu]
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
MFMA_PEAK_TFLOPS = 2500.0      # dense fp16 matrix-core peak, published
CACHE_BYTES = 256 << 20        # last-level (Infinity) cache
KIB = 1024
# HBM bytes per launch of each kernel group, measured OFFLINE with `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`
# (KiB per dispatch, scaled by what the same counters read for a plain copy of known size: FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0): read from the text summary of those runs under profiles/ (columns: workload, group, bytes,
# kernels); null where the file or the group is missing.  Not measured by this script.
TRAFFIC_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic_per_launch_group.txt")


def load_offline_traffic():
    table = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                p = line.split()
                if len(p) >= 3 and not line.startswith("#"):
                    table.setdefault(p[0], {})[p[1]] = float(p[2])
    except OSError:
        pass
    return table


OFFLINE_TRAFFIC = load_offline_traffic()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ---------------------------------------------------------------------------------------------
# byte and flop models
# ---------------------------------------------------------------------------------------------
def group_bytes(w: wl.Workload):
    """Algorithmic bytes (user-visible tensors only) of each launch group taken as a unit."""
    s = wl.DTYPE_BYTES[w.dtype]
    E = w.B * w.H * w.N
    hn = 4 * w.H * w.N + 4 * w.H
    fwd_b, bwd_b = wl.algorithmic_bytes(w.B, w.H, w.N, w.dtype)
    return {"kspec": 0,                       # its read of k is charged to fwd
            "fwd": fwd_b,                     # u in, y out, k and D in
            "bwd": bwd_b,                     # dy, u in; du out; k in, dk out; D in, dD out
            "bwd_dk": 2 * E * s + hn,         # dy, u in; dk, dD out
            "bwd_du": 2 * E * s + hn}         # dy in, du out; k, D in


def executed_mfma_flops(w: wl.Workload):
    """Matrix-core flops the kernels issue for one step (model of the factorisation, dense 16x16x32 blocks,
    two instructions per 16x16 complex tile and stage, 16384 flop each): per 256-point tile a forward or an
    inverse half transform costs 8 instructions on the cooperative kernels (four stages), 6 on the
    wave-autonomous ones (three stages).  Half transforms per row pair: forward 2, backward 3 where one kernel
    serves du, dk and dD (up to 4096 points) else 4; per head: spectrum 1, dk's inverse 1."""
    if w.dtype == wl.F32:
        return 0.0
    L = 2 * w.N
    npairs = (w.B + 1) // 2
    per_half = (6 if L <= 4096 else 8) * 16384 * (L / 256)
    bwd_halves = 3 if L <= 4096 else 4
    fwd_halves, head_halves = 2.0, 2.0
    if L > 32768 and w.B == 1:
        # a batch of one row: the multi-pass kernels compute the chunks 0 .. R/2 of R only (Hermitian spectrum);
        # the convolutions split into R = L / 32768 chunks, dk into 2R chunks of 16384 points
        R = L // 32768
        fc, fd = (R / 2 + 1) / R, (R + 1) / (2 * R)
        fwd_halves, bwd_halves, head_halves = 2 * fc, 2 * fc + 2 * fd, 1 + fd
    return w.H * (npairs * (fwd_halves + bwd_halves) + head_halves) * per_half


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


def timed(torch, steps, fn):
    """ms per step of `steps` calls of fn(i) between two events on the launch stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def run_workload(key, steps, warmup, lc, torch):
    w = wl.WORKLOADS[key]
    S = Sets(w, lc, torch)
    plan = lc.longconv_plan_string(w.N, w.dtype)
    one_kernel_bwd = "kernel=wave" in plan            # du, dk, dD of a call come from one kernel
    gb = group_bytes(w)
    groups = ["kspec", "fwd"] + (["bwd"] if one_kernel_bwd else ["bwd_dk", "bwd_du"])

    def step(i, cold=True):
        j = i % S.nsets
        if cold:
            lc.longconv_kspec_compute(S.k, S.D, S.kspec, w.dtype, S.ws)
        lc.longconv_fwd(S.u[j], S.k, S.D, S.y[j], S.ws, kspec=S.kspec)
        lc.longconv_bwd(S.dy[j], S.u[j], S.k, S.D, S.du[j], S.dk, S.dD, S.ws, kspec=S.kspec)

    def step_marked(i, m):
        j = i % S.nsets
        m[0].record()
        lc.longconv_kspec_compute(S.k, S.D, S.kspec, w.dtype, S.ws)
        m[1].record()
        lc.longconv_fwd(S.u[j], S.k, S.D, S.y[j], S.ws, kspec=S.kspec)
        m[2].record()
        if one_kernel_bwd:
            lc.longconv_bwd(S.dy[j], S.u[j], S.k, S.D, S.du[j], S.dk, S.dD, S.ws, kspec=S.kspec)
            m[3].record()
        else:       # the same kernels the single call launches, with an event between them
            lc.longconv_bwd(S.dy[j], S.u[j], S.k, S.D, None, S.dk, S.dD, S.ws, kspec=S.kspec)
            m[3].record()
            lc.longconv_bwd(S.dy[j], S.u[j], S.k, S.D, S.du[j], None, None, S.ws, kspec=S.kspec)
            m[4].record()

    for i in range(warmup):
        step(i)
    # ---- headline region: exactly `steps` cold-spectrum steps, HBM-cold buffers, nothing in between
    t0 = time.perf_counter()
    step_ms = timed(torch, steps, lambda i: step(warmup + i))
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    # ---- per-call durations
    ng = len(groups)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(ng + 1)] for _ in range(steps)]
    for i in range(steps):
        step_marked(warmup + steps + i, marks[i])
    torch.cuda.synchronize()
    seg = np.array([[m[a].elapsed_time(m[a + 1]) for a in range(ng)] for m in marks])   # ms
    # ---- warm spectrum (cached), still HBM-cold buffers
    warm_ms = timed(torch, steps, lambda i: step(i, cold=False))
    # ---- cache-hot: one buffer set only
    S_n = S.nsets
    S.nsets = 1
    for i in range(3):
        step(i)
    hot_ms = timed(torch, steps, lambda i: step(i))
    S.nsets = S_n

    fwd_b, bwd_b = gb["fwd"], gb["bwd"]
    tot_b = fwd_b + bwd_b
    ff, bf = wl.algorithmic_flops(w.B, w.H, w.N)
    mf = executed_mfma_flops(w)
    segments = {n: {"ms_mean": float(seg[:, i].mean()), "ms_median": float(np.median(seg[:, i])),
                    "ms_min": float(seg[:, i].min()), "algorithmic_bytes": gb[n],
                    "GBps": (gb[n] / (seg[:, i].mean() * 1e-3) / 1e9) if gb[n] else None}
                for i, n in enumerate(groups)}
    dom = max((n for n in groups if gb[n]), key=lambda n: segments[n]["ms_mean"])
    res = {
        "workload": w.name, "B": w.B, "H": w.H, "N": w.N, "io": wl.DTYPE_NAMES[w.dtype], "plan": plan,
        "buffer_sets": S.nsets, "steps": steps,
        "ms_per_step": float(step_ms), "wall_ms_per_step": wall_ms,
        "ms_per_step_instrumented_mean": float(seg.sum(axis=1).mean()),
        "ms_per_step_instrumented_median": float(np.median(seg.sum(axis=1))),
        "ms_per_step_instrumented_min": float(seg.sum(axis=1).min()),
        "bytes_per_step": tot_b, "GBps": tot_b / (step_ms * 1e-3) / 1e9,
        "pct_hbm_roofline": 100.0 * tot_b / (step_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "warm_spectrum": {"ms_per_step": float(warm_ms), "GBps": tot_b / (warm_ms * 1e-3) / 1e9,
                          "pct_hbm_roofline": 100.0 * tot_b / (warm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "cache_hot_same_buffers": {"ms_per_step": float(hot_ms), "GBps": tot_b / (hot_ms * 1e-3) / 1e9,
                                   "note": "one buffer set reused every step: data served by the last-level cache, not HBM"},
        "fwd_ms": segments["fwd"]["ms_mean"],
        "fwd_pct_hbm_roofline": 100.0 * segments["fwd"]["GBps"] / HBM_PEAK_GBS,
        "segments": segments,
        "TFLOPs_algorithmic": (ff + bf) / (step_ms * 1e-3) / 1e12,
        "mfma_executed": {"TFLOPs": mf / (step_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS,
                          "pct_of_peak": 100.0 * mf / (step_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                          "flops_per_step_model": mf},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": segments[dom]["GBps"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": segments[dom]["GBps"] / HBM_PEAK_GBS,
                     "traffic": OFFLINE_TRAFFIC.get(w.name, {}).get(dom),
                     "traffic_source": ("offline rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, profiles/hbm_traffic_per_launch_group.txt"
                                        if OFFLINE_TRAFFIC.get(w.name, {}).get(dom) else None),
                     "algorithmic_bytes_per_launch": gb[dom],
                     "avg_launch_ms": segments[dom]["ms_mean"]},
    }
    del S
    torch.cuda.empty_cache()
    return res


def copy_bandwidth(torch, nbytes=1 << 30, reps=10):
    """Plain device-to-device copy of 1 GiB, read + written bytes per second."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    ms = timed(torch, reps, lambda i: dst.copy_(src))
    del src, dst
    torch.cuda.empty_cache()
    return 2 * nbytes / (ms * 1e-3) / 1e9


def copy_probe(torch):
    """Reference dispatches for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters (only with --copy-probe):
    a contiguous 64 MiB device copy (whole 128-byte lines), and a copy that reads every other 64-byte segment of a
    64 MiB buffer (32 MiB read in 64-byte requests, 32 MiB written)."""
    n = (64 << 20) // 4
    src = torch.zeros(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    half = torch.empty(n // 2, dtype=torch.float32, device="cuda")
    for _ in range(3):
        dst.copy_(src)
        half.view(-1, 16).copy_(src.view(-1, 2, 16)[:, 0, :])
    torch.cuda.synchronize()


def cpu_baseline(key):
    """The float64 oracle, as it stands, on the host cores: whole workload if it is a few seconds of
    work, otherwise all batch rows of a subset of heads (cost is linear in heads)."""
    import oracle
    w = wl.WORKLOADS[key]
    macs_per_head = 3 * w.B * w.N * w.N / 2          # fwd + du + dk
    budget = 15.0 * 50e9                             # about 15 s at ~50 GMAC/s
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
    ap.add_argument("--workload", default="3", choices=list(wl.WORKLOADS))
    ap.add_argument("--also", default="4a,2", help="comma list of further workloads reported under 'targets'")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run two copies of known size (reference for scaling rocprofv3 byte counters)")
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
    copy_gbs = copy_bandwidth(torch)
    if a.copy_probe:
        copy_probe(torch)

    res = run_workload(a.workload, a.steps, a.warmup, lc, torch)
    log(json.dumps(res, indent=1))
    w = wl.WORKLOADS[a.workload]
    out = {
        "metric": "long-conv fwd+bwd ms, effective GB/s and % HBM roofline at BxHxN",
        "value": res["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # arithmetic type of the transforms: fp16 matrix-core operands with fp32 accumulation for fp16 and bf16
        # I/O (bf16 inputs are converted on load), fp32 for fp32 I/O; the I/O dtype is config.io
        "dtype": "f32" if w.dtype == wl.F32 else "f16", "data": "synthetic",
        "config": {"workload": res["workload"], "B": res["B"], "H": res["H"], "N": res["N"], "io": res["io"],
                   "step": "kspec+fwd+bwd(du,dk,dD), cold spectrum, HBM-cold buffers", "plan": res["plan"],
                   "buffer_sets": res["buffer_sets"]},
        "pct_hbm_roofline": res["pct_hbm_roofline"],
        "pct_of_copy_bandwidth": 100.0 * res["GBps"] / copy_gbs,
        "copy_bandwidth_GBps": copy_gbs,
        "ms_per_step_median_instrumented": res["ms_per_step_instrumented_median"],
        "ms_per_step_min_instrumented": res["ms_per_step_instrumented_min"],
        "fwd_ms": res["fwd_ms"], "fwd_pct_hbm_roofline": res["fwd_pct_hbm_roofline"],
        "warm_spectrum": res["warm_spectrum"], "cache_hot_same_buffers": res["cache_hot_same_buffers"],
        "TFLOPs_algorithmic": res["TFLOPs_algorithmic"], "mfma_executed": res["mfma_executed"],
        "segments": res["segments"],
        "roofline": res["roofline"],
    }
    targets = []
    for key in [k for k in a.also.split(",") if k and k != a.workload]:
        r = run_workload(key, max(20, a.steps // 2), max(5, a.warmup // 2), lc, torch)
        log(json.dumps(r, indent=1))
        targets.append({k: r[k] for k in ("workload", "plan", "steps", "ms_per_step", "GBps", "pct_hbm_roofline", "fwd_ms",
                                          "fwd_pct_hbm_roofline", "warm_spectrum", "cache_hot_same_buffers", "mfma_executed",
                                          "segments", "roofline")})
    out["targets"] = targets
    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(a.workload)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
