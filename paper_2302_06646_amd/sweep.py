"""Length sweep and block-size-table shape on one MI355X: `python -m paper_2302_06646_amd.sweep [--quick]`;
`--learned` times the learned Butterfly extension against the fixed path instead (the shape of the paper's table of
learnable block sizes: block size 16 against the fixed Butterfly, as a speed ratio); `--blocks` runs the table of
block sizes (2 ... 32 points per block at N = 4096, B = 128, H = 32) with the study kernel.

Two measurements that mirror the paper's efficiency experiments (Section 5.4 runtime figure: one layer, batch 32,
128 heads, N = 1K ... 128K, against the FFT-library convolution; Table of block sizes: N = 4096, B = 128, H = 32),
on synthetic data:

  * forward time of this library (cached spectrum, and with the spectrum recomputed) against the same
    convolution through torch.fft (rocFFT: rfft of the padded fp32 copy, multiply, irfft, truncate, skip term),
    the analogue of the paper's cuFFT baseline.  Context only: the torch.fft route is not the oracle and is
    never on the product path.
  * forward, backward and whole-step time at the block-size table's shape, with the factorisation the plan
    picks (the library runs 16-point blocks on the matrix cores and shorter last blocks as block-diagonal
    16 x 16 matrices).

Each timing: rotating buffer sets (HBM-cold), `steps` calls between two events on the launch stream.
Prints a markdown table and one JSON line per row.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

import paper_2302_06646_amd as lc

F16 = lc.F16


def _timed(steps, fn):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps * 1e3      # microseconds


def _sets(B, H, N, want_bytes=640 << 20, backward=False):
    per = (4 if backward else 2) * B * H * N * 2
    n = max(2, min(8, -(-want_bytes // per)))
    g = torch.Generator(device="cuda").manual_seed(N)
    mk = lambda: torch.randn((B, H, N), generator=g, device="cuda", dtype=torch.float32).to(torch.float16)
    return n, [mk() for _ in range(n)], [torch.empty((B, H, N), device="cuda", dtype=torch.float16) for _ in range(n)]


def fft_conv_time(u_sets, k, D, steps):
    """The FFT-library convolution: y = irfft(rfft(u, 2N) * rfft(k, 2N))[:N] + D u, fp32 transforms of fp16 data,
    kernel spectrum precomputed (as for the cached-spectrum column)."""
    N = k.shape[-1]
    kf = torch.fft.rfft(k, n=2 * N)
    outs = [torch.empty_like(u) for u in u_sets]

    def fn(i):
        j = i % len(u_sets)
        u = u_sets[j].float()
        y = torch.fft.irfft(torch.fft.rfft(u, n=2 * N) * kf, n=2 * N)[..., :N] + D[None, :, None] * u
        outs[j].copy_(y)
    fn(0)
    return _timed(steps, fn)


def sweep_row(B, H, N, steps):
    io = F16
    nsets, us, ys = _sets(B, H, N)
    k = torch.randn(H, N, device="cuda") / N ** 0.5
    D = torch.randn(H, device="cuda")
    ks = lc.new_kspec(H, N, io)
    ws = lc.new_workspace(B, H, N, io, False)
    lc.longconv_kspec_compute(k, D, ks, io, ws)
    warm = lambda i: lc.longconv_fwd(us[i % nsets], k, D, ys[i % nsets], ws, kspec=ks)
    cold = lambda i: lc.longconv_fwd(us[i % nsets], k, D, ys[i % nsets], ws)
    for i in range(3):
        warm(i); cold(i)
    t_warm, t_cold = _timed(steps, warm), _timed(steps, cold)
    t_fft = fft_conv_time(us, k, D, max(3, steps // 4))
    bytes_fwd = 2 * B * H * N * 2 + 4 * H * N + 4 * H
    return {"B": B, "H": H, "N": N, "plan": lc.longconv_plan_string(N, io), "fwd_cached_spectrum_us": t_warm,
            "fwd_with_spectrum_us": t_cold, "torch_fft_conv_us": t_fft, "speedup_vs_fft_library": t_fft / t_warm,
            "fwd_GBps": bytes_fwd / t_warm / 1e3, "pct_hbm_roofline": 100 * bytes_fwd / t_warm / 1e3 / 8000.0}


def table_shape(B, H, N, steps):
    io = F16
    nsets, us, ys = _sets(B, H, N, backward=True)
    _, dys, dus = _sets(B, H, N, backward=True)
    k = torch.randn(H, N, device="cuda") / N ** 0.5
    D = torch.randn(H, device="cuda")
    dk, dD = torch.empty_like(k), torch.empty_like(D)
    ks = lc.new_kspec(H, N, io)
    ws = lc.new_workspace(B, H, N, io, True)
    kspec = lambda i: lc.longconv_kspec_compute(k, D, ks, io, ws)
    fwd = lambda i: lc.longconv_fwd(us[i % nsets], k, D, ys[i % nsets], ws, kspec=ks)
    bwd = lambda i: lc.longconv_bwd(dys[i % nsets], us[i % nsets], k, D, dus[i % nsets], dk, dD, ws, kspec=ks)
    for i in range(3):
        kspec(i); fwd(i); bwd(i)
    t = {"kspec_us": _timed(steps, kspec), "fwd_us": _timed(steps, fwd), "bwd_us": _timed(steps, bwd)}
    t_fft = fft_conv_time(us, k, D, max(3, steps // 4))
    L = 2 * N
    # executed matrix-core flops of the forward pass: 8 instructions of 16384 flop per 256-point tile and half
    # transform (four 16-point stages, the last one block-diagonal), two half transforms per row pair
    mf = H * ((B + 1) // 2) * 2 * 8 * 16384 * (L / 256)
    return {"B": B, "H": H, "N": N, "plan": lc.longconv_plan_string(N, io), **t, "torch_fft_conv_fwd_us": t_fft,
            "fwd_executed_mfma_GFLOP": mf / 1e9, "fwd_mfma_TFLOPs": mf / t["fwd_us"] / 1e6,
            "fwd_mfma_pct_of_peak": 100 * mf / t["fwd_us"] / 1e6 / 2500.0}


def dft_blocks(H, N):
    """[H, 3, 16, 16, 2] float32 blocks that make the learned path the plain FFT convolution, and their conjugates."""
    import numpy as np
    A = np.zeros((H, 3, 16, 16, 2), dtype=np.float32)
    for s, r in enumerate((16, 16, 2 * N // 256)):
        F = np.exp(-2j * np.pi * np.outer(np.arange(r), np.arange(r)) / r)
        A[:, s, :r, :r, 0], A[:, s, :r, :r, 1] = F.real, F.imag
    Af = torch.from_numpy(A).cuda()
    Ai = Af.clone()
    Ai[..., 1] *= -1
    return Af, Ai


def learned_row(B, H, N, steps):
    """Fixed path against the learned Butterfly extension, bf16 rows, forward and backward (all gradients)."""
    io, td = lc.BF16, torch.bfloat16
    nsets = 4
    g = torch.Generator(device="cuda").manual_seed(N)
    mk = lambda: torch.randn((B, H, N), generator=g, device="cuda", dtype=torch.float32).to(td)
    us, dys = [mk() for _ in range(nsets)], [mk() for _ in range(nsets)]
    y, du = torch.empty_like(us[0]), torch.empty_like(us[0])
    k = torch.randn(H, N, device="cuda") / N ** 0.5
    D = torch.randn(H, device="cuda")
    dk, dD = torch.empty_like(k), torch.empty_like(D)
    Af, Ai = dft_blocks(H, N)
    dAf, dAi = torch.empty_like(Af), torch.empty_like(Ai)
    shat = torch.empty(H, 2 * N, 2, device="cuda")
    dshat = torch.empty_like(shat)
    wsl = torch.empty(lc.longconv_lbfly_workspace_bytes(B, H, N, io), dtype=torch.uint8, device="cuda")
    ws = lc.new_workspace(B, H, N, io, True)
    fns = {
        "fixed_fwd_us": lambda i: lc.longconv_fwd(us[i % nsets], k, D, y, ws),
        "fixed_bwd_us": lambda i: lc.longconv_bwd(dys[i % nsets], us[i % nsets], k, D, du, dk, dD, ws),
        "learned_spectrum_us": lambda i: lc.longconv_lbfly_spectrum(k, D, shat),
        "learned_fwd_us": lambda i: lc.longconv_lbfly_fwd(us[i % nsets], shat, Af, Ai, y),
        "learned_bwd_us": lambda i: lc.longconv_lbfly_bwd(dys[i % nsets], us[i % nsets], shat, Af, Ai, du, dshat, dAf,
                                                           dAi, wsl),
        "learned_spectrum_bwd_us": lambda i: lc.longconv_lbfly_spectrum_bwd(dshat, dk, dD),
    }
    r = {"B": B, "H": H, "N": N, "dtype": "bf16"}
    for name, fn in fns.items():
        for i in range(3):
            fn(i)
        r[name] = _timed(steps, fn)
    fixed = r["fixed_fwd_us"] + r["fixed_bwd_us"]
    learned = sum(r[n] for n in fns if n.startswith("learned"))
    r["speed_ratio_learned_over_fixed"] = fixed / learned
    # bytes of the rows the step has to move: u and y forward, dy, u and du backward
    r["learned_step_GBps"] = 5 * B * H * N * 2 / learned / 1e3
    # matrix-core work of the learned step: two instructions of 16384 flop per 256-point tile and block product;
    # 6 block products forward, 12 + 1 (the transform again) backward, 6 block gradients
    r["learned_step_mfma_TFLOPs"] = B * H * (2 * N / 256) * (6 + 13 + 6) * 2 * 16384 / learned / 1e6
    return r


def block_sizes(B, H, N, steps):
    """The paper's table of block sizes at its shape (fp16 rows): forward time of the study kernel with DFT blocks of
    2, 4, 8, 16 points (every block run as one 16 x 16 matrix product), 32 points (one 32 x 32 product), 64 and 256
    points (dense products in 32 x 32 tiles; the bits a whole number of such blocks leaves over run as one narrower
    stage), and the matrix-core work it executes."""
    td = torch.float16
    nsets = 4
    g = torch.Generator(device="cuda").manual_seed(N)
    us = [torch.randn((B, H, N), generator=g, device="cuda", dtype=torch.float32).to(td) for _ in range(nsets)]
    y = torch.empty_like(us[0])
    k = torch.randn(H, N, device="cuda") / N ** 0.5
    D = torch.randn(H, device="cuda")
    shat = torch.empty(H, 2 * N, 2, device="cuda")
    lc.longconv_lbfly_spectrum(k, D, shat)
    LG = (2 * N).bit_length() - 1

    def stage_flop_per_point(bits):
        # matrix-core flop per point of one stage whose digit has `bits` bits, as the study kernels run it:
        # up to 4 bits: two instructions of 16384 flop per 256-point tile; 5 bits: eight of 32768 flop per 1024-point
        # tile; r = 64, 256: the dense 2r x 2r real product, 8 r flop per point
        if bits <= 4:
            return 2 * 16384 / 256
        if bits == 5:
            return 8 * 32768 / 1024
        return 8 * (1 << bits)

    rows = []
    for log2r in (1, 2, 3, 4, 5, 6, 8):
        fn = lambda i: lc.longconv_blocksize_fwd(us[i % nsets], shat, y, log2r)
        for i in range(3):
            fn(i)
        t = _timed(steps, fn)
        stages = -(-LG // log2r)
        digits = [log2r] * (stages - 1) + [LG - log2r * (stages - 1)]
        # forward and inverse chain, one complex sequence per real row
        # (the 32-point kernel runs its last, narrower digit on the 32-wide tile as well)
        gflop = B * H * 2 * N * 2 * sum(stage_flop_per_point(5 if log2r == 5 else b) for b in digits) / 1e9
        # what the same stages would cost with blocks of exactly r points: 8 r flop per point and stage
        nominal = B * H * 2 * N * 2 * stages * 8 * (1 << log2r) / 1e9   # (the last, narrower stage counted as a full one)
        rows.append({"B": B, "H": H, "N": N, "block": 1 << log2r, "stages_each_way": stages, "fwd_us": t,
                     "executed_mfma_GFLOP": gflop, "nominal_GFLOP": nominal, "mfma_TFLOPs": gflop / t * 1e3,
                     "mfma_pct_of_peak": 100 * gflop / t * 1e3 / 2500.0})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="fewer steps and lengths")
    ap.add_argument("--learned", action="store_true", help="learned Butterfly extension against the fixed path")
    ap.add_argument("--blocks", action="store_true", help="the table of block sizes: 2 ... 64 and 256 at N=4096, B=128, H=32")
    a = ap.parse_args()
    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        sys.exit(1)
    lc.longconv_init()
    steps = 10 if a.quick else 30
    if a.blocks:
        rows = block_sizes(128, 32, 4096, steps)
        print("| block size | stages each way | fwd (us) | executed MFMA GFLOP | GFLOP at r-point blocks | TFLOP/s | % of 2.5 PFLOP/s |")
        print("|---|---|---|---|---|---|---|")
        for r in rows:
            print(f"| {r['block']} | {r['stages_each_way']} | {r['fwd_us']:.1f} | {r['executed_mfma_GFLOP']:.1f} | "
                  f"{r['nominal_GFLOP']:.1f} | {r['mfma_TFLOPs']:.0f} | {r['mfma_pct_of_peak']:.1f} |")
        for r in rows:
            print(json.dumps(r))
        return
    if a.learned:
        shapes = [(16, 768, 1024)] if a.quick else [(16, 768, 1024), (64, 256, 1024), (64, 1024, 256), (64, 1024, 2048)]
        rows = [learned_row(B, H, N, steps) for (B, H, N) in shapes]
        print("| B, H, N | fixed fwd / bwd (us) | learned spectrum / fwd / bwd / spectrum bwd (us) | speed ratio | "
              "learned step GB/s | MFMA TFLOP/s |")
        print("|---|---|---|---|---|---|")
        for r in rows:
            print(f"| {r['B']}, {r['H']}, {r['N']} | {r['fixed_fwd_us']:.1f} / {r['fixed_bwd_us']:.1f} | "
                  f"{r['learned_spectrum_us']:.1f} / {r['learned_fwd_us']:.1f} / {r['learned_bwd_us']:.1f} / "
                  f"{r['learned_spectrum_bwd_us']:.1f} | {r['speed_ratio_learned_over_fixed']:.2f}x | "
                  f"{r['learned_step_GBps']:.0f} | {r['learned_step_mfma_TFLOPs']:.1f} |")
        for r in rows:
            print(json.dumps(r))
        return
    lengths = [1024, 16384, 131072] if a.quick else [1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072]
    rows = [sweep_row(32, 128, N, steps) for N in lengths]
    print("| N | plan | fwd, cached spectrum (us) | fwd + spectrum (us) | torch.fft conv (us) | speed-up | GB/s | % of 8 TB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['N']} | {r['plan'].split('digits=')[-1]} | {r['fwd_cached_spectrum_us']:.1f} | {r['fwd_with_spectrum_us']:.1f} | "
              f"{r['torch_fft_conv_us']:.1f} | {r['speedup_vs_fft_library']:.1f}x | {r['fwd_GBps']:.0f} | {r['pct_hbm_roofline']:.1f} |")
    t = table_shape(128, 32, 4096, steps)
    print()
    print("| shape | plan | kspec (us) | fwd (us) | bwd (us) | torch.fft conv fwd (us) | fwd executed MFMA GFLOP | TFLOP/s | % of 2.5 PFLOP/s |")
    print("|---|---|---|---|---|---|---|---|---|")
    print(f"| B=128 H=32 N=4096 fp16 | {t['plan'].split('digits=')[-1]} | {t['kspec_us']:.1f} | {t['fwd_us']:.1f} | {t['bwd_us']:.1f} | "
          f"{t['torch_fft_conv_fwd_us']:.1f} | {t['fwd_executed_mfma_GFLOP']:.1f} | {t['fwd_mfma_TFLOPs']:.0f} | {t['fwd_mfma_pct_of_peak']:.1f} |")
    for r in rows + [t]:
        print(json.dumps(r))


if __name__ == "__main__":
    main()
