"""bf16 rows far outside fp16's exponent range (the transforms carry fp16 between their stages): tiny gradients,
large activations, rows of one head that differ by many orders of magnitude.  Every row (y, du) and every head
(dk, dD) must meet the same bound as data of order one."""
import dataclasses

import numpy as np
import pytest

import workloads as wl
from gpu_harness import check_full

pytestmark = pytest.mark.gpu


def scaled_inputs(N, B, H, u_scale, dy_scale, k_scale=None, D_scale=None, seed=0):
    """Workload-2 style bf16 inputs; row (b,h) of u is multiplied by u_scale[b,h] (broadcast), likewise dy; head h
    of k by k_scale[h] and D[h] by D_scale[h]; u and dy are rounded to bf16 again afterwards."""
    w = wl.Workload(2, B, H, N, wl.BF16, "squash_pool")
    inp = wl.generate(w, seed_extra=seed)
    us = np.broadcast_to(np.asarray(u_scale, dtype=np.float64), (B, H))[:, :, None]
    ds = np.broadcast_to(np.asarray(dy_scale, dtype=np.float64), (B, H))[:, :, None]
    u_s, u_v = wl.quantize((inp.u * us).astype(np.float32), wl.BF16)
    dy_s, dy_v = wl.quantize((inp.dy * ds).astype(np.float32), wl.BF16)
    k, D = inp.k, inp.D
    if k_scale is not None:
        k = (k.astype(np.float64) * np.asarray(k_scale, dtype=np.float64)[:, None]).astype(np.float32)
    if D_scale is not None:
        D = (D.astype(np.float64) * np.asarray(D_scale, dtype=np.float64)).astype(np.float32)
    return dataclasses.replace(inp, u_store=u_s, dy_store=dy_s, u=u_v, dy=dy_v, k=k, D=D)


LENGTHS = [256, 512, 1024, 2048, 4096, 8192, 16384]      # every single-pass plan


@pytest.mark.parametrize("N", LENGTHS)
def test_tiny_gradients_and_large_activations(N):
    # dy ~ N(0, 1e-10) (standard deviation 1e-5), u ~ N(0, 1e6)
    check_full(scaled_inputs(N, 5, 3, 1e3, 1e-5), label=f"u 1e3, dy 1e-5, N={N}")


@pytest.mark.parametrize("N", LENGTHS)
def test_rows_of_one_head_at_very_different_magnitudes(N):
    B, H = 6, 2
    # every row either of order one or at least a factor 100 away from it (rows that differ by less than the
    # width of the unscaled band, 2^6, share one fp16 scale inside a pair: their error is relative to the larger)
    rng = np.random.default_rng(7 + N)
    us = 10.0 ** (rng.choice([-1, 1], size=(B, H)) * rng.uniform(2, 8, size=(B, H)))
    ds = 10.0 ** np.where(rng.random((B, H)) < 0.7, rng.uniform(-12, -3, size=(B, H)), rng.uniform(2, 4, size=(B, H)))
    us[0, 0], ds[0, 0] = 1.0, 1.0            # rows inside the band next to the others
    us[3, 1], ds[2, 0] = 1.0, 1.0
    check_full(scaled_inputs(N, B, H, us, ds, seed=1), label=f"mixed magnitudes, N={N}")


@pytest.mark.parametrize("N", [32768, 65536])
def test_multi_pass_lengths_scale_per_head(N):
    # the multi-pass plans rescale per head (all rows of a head by one power of two): uniform tiny gradients and
    # large activations, and heads at very different magnitudes
    check_full(scaled_inputs(N, 3, 2, 1e3, 1e-5), label=f"u 1e3, dy 1e-5, N={N}")
    us = np.array([[1e-6, 3e4]])
    ds = np.array([[2e-9, 1.0]])
    check_full(scaled_inputs(N, 2, 2, us, ds, seed=2), label=f"heads at different magnitudes, N={N}")
