"""Seeded random small shapes through every entry point of the data path: batch sizes that are odd, one or large
against the head count (pairs dealt to several workgroups), single heads, every length up to 16384 and one
multi-pass length, all three I/O dtypes; forward, backward and the gated layer against the oracles."""
import numpy as np
import pytest

import workloads as wl
from gpu_harness import check_full
import test_gated_gpu as tg
from oracle import gated

pytestmark = pytest.mark.gpu

_rng = np.random.default_rng(20230213)
_LENGTHS = [256, 512, 1024, 2048, 4096, 8192, 16384]
CASES = []
for _ in range(18):
    CASES.append((int(_rng.choice(_LENGTHS)), int(_rng.choice([wl.F32, wl.F16, wl.BF16], p=[0.2, 0.4, 0.4])),
                  int(_rng.integers(1, 10)), int(_rng.integers(1, 6)), int(_rng.integers(0, 1000))))
CASES += [(32768, wl.F16, 3, 1, 5), (65536, wl.BF16, 2, 2, 6)]


@pytest.mark.parametrize("N,io,B,H,seed", CASES)
def test_random_shape(N, io, B, H, seed):
    kind = {wl.F32: "decay256", wl.F16: "decay_alpha_squash", wl.BF16: "squash_pool"}[io]
    inp = wl.generate(wl.Workload(7, B, H, N, io, kind), seed_extra=seed)
    check_full(inp, label=f"random N={N} io={wl.DTYPE_NAMES[io]} B={B} H={H}")


@pytest.mark.parametrize("N,io,B,H,seed", CASES[::3])
def test_random_shape_gated(N, io, B, H, seed):
    inp, g_s, g_v = tg._inputs(N, io, B, H, seed)
    y, du, dk, dD, dg = tg._run(inp, g_s)
    k64, D64 = inp.k.astype(np.float64), inp.D.astype(np.float64)
    ry = gated.gated_fwd(inp.u, k64, D64, g_v)
    rdu, rdk, rdD, rdg = gated.gated_bwd(inp.dy, g_v, inp.u, k64, D64)
    tol = 1e-5 if io == wl.F32 else 3e-3
    for name, a, b in (("y", y, ry), ("du", du, rdu), ("dk", dk, rdk), ("dg", dg, rdg), ("dD", dD, rdD)):
        e = wl.rel_l2(a, b)
        assert np.isfinite(e) and e <= (1e-5 if name == "dD" else tol), (name, e)
