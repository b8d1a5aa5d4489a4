"""bf16 rows far outside fp16's exponent range (the transforms carry fp16 between their stages): tiny gradients,
large activations, rows of one head that differ by many orders of magnitude.  Every row (y, du) and every head
(dk, dD) must meet the same bound as data of order one."""
import dataclasses

import numpy as np
import pytest

import workloads as wl
from gpu_harness import check_full

pytestmark = pytest.mark.gpu


def scaled_inputs(N, B, H, u_scale, dy_scale, k_scale=None, D_scale=None, seed=0, dtype=wl.BF16):
    """Workload-2 style inputs (bf16 unless said otherwise); row (b,h) of u is multiplied by u_scale[b,h]
    (broadcast), likewise dy; head h of k by k_scale[h] and D[h] by D_scale[h]; u and dy are rounded to the I/O
    dtype again afterwards."""
    w = wl.Workload(2, B, H, N, dtype, "squash_pool")
    inp = wl.generate(w, seed_extra=seed)
    us = np.broadcast_to(np.asarray(u_scale, dtype=np.float64), (B, H))[:, :, None]
    ds = np.broadcast_to(np.asarray(dy_scale, dtype=np.float64), (B, H))[:, :, None]
    u_s, u_v = wl.quantize((inp.u * us).astype(np.float32), dtype)
    dy_s, dy_v = wl.quantize((inp.dy * ds).astype(np.float32), dtype)
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


# The stored spectrum is fp16: a head whose spectrum lies outside fp16's comfortable range is stored with a power of
# two taken out, which the convolution kernels give back where they pack their output.  One wave length, the
# cooperative lengths and two multi-pass lengths; every row of every head to the bound of data of order one.
@pytest.mark.parametrize("N", [256, 1024, 4096, 16384, 65536, 131072])
def test_kernels_of_any_magnitude_bf16(N):
    B = 3 if N <= 16384 else 2
    ks = np.array([2.0 ** -20, 2.0 ** 20, 1.0, 2.0 ** -30, 2.0 ** 12, 1e-3, 3e4])
    Ds = np.array([2.0 ** -20, 2.0 ** 20, 1.0, 1.0, 2.0 ** -5, 1e3, 3e-4])      # skip term with, above and below the kernel
    H = len(ks) if N <= 16384 else 4
    check_full(scaled_inputs(N, B, H, 1.0, 1.0, k_scale=ks[:H], D_scale=Ds[:H], seed=3), label=f"kernel magnitudes, N={N}")


@pytest.mark.parametrize("N", [512, 8192, 32768])
def test_kernels_of_other_magnitudes_fp16(N):
    # fp16 rows and outputs have to stay inside fp16's own range: heads at 2^-9 and 2^9 with rows of order one
    ks = np.array([2.0 ** -9, 2.0 ** 9, 1.0, 2.0 ** -6])
    check_full(scaled_inputs(N, 3, 4, 1.0, 1.0, k_scale=ks, D_scale=ks, seed=4, dtype=wl.F16), label=f"kernel magnitudes fp16, N={N}")


def test_kernel_magnitude_with_rows_out_of_band():
    # both rescalings at once on a single-pass plan: tiny gradients, large activations and kernels far from one
    ks = np.array([2.0 ** -18, 2.0 ** 15, 1.0])
    check_full(scaled_inputs(2048, 4, 3, 1e3, 1e-5, k_scale=ks, D_scale=ks, seed=5), label="rows and kernels out of range, N=2048")
    check_full(scaled_inputs(16384, 3, 3, 1e3, 1e-5, k_scale=ks, D_scale=ks, seed=6), label="rows and kernels out of range, N=16384")


@pytest.mark.parametrize("N", [256, 1024, 2048, 8192, 16384])
def test_rows_of_a_pair_a_few_times_apart(N):
    # the two rows of a pair share one complex transform, so the rounding of the larger is an error of the smaller:
    # rows that differ by a factor of four and more have to be scaled one by one even when both are of "ordinary"
    # size, and a row of ordinary size next to one that needs scaling anyway is scaled with it
    B, H = 8, 3
    us = np.ones((B, H)); ds = np.ones((B, H))
    us[0:2, 0] = [0.1, 1.0]; us[2:4, 0] = [3.5, 0.09]; us[4:6, 0] = [0.3, 1e4]; us[6:8, 0] = [0.26, 3.9]
    ds[0:2, 0] = [1.0, 0.08]; ds[2:4, 0] = [0.3, 3e-6]; ds[4:6, 0] = [2.0, 0.5]; ds[6:8, 0] = [0.07, 0.9]
    rng = np.random.default_rng(11 + N)
    us[:, 1] = 10.0 ** rng.uniform(-1.2, 1.2, size=B); ds[:, 1] = 10.0 ** rng.uniform(-1.2, 1.2, size=B)
    us[:, 2] = 10.0 ** rng.uniform(-6, 6, size=B); ds[:, 2] = 10.0 ** rng.uniform(-9, 3, size=B)
    check_full(scaled_inputs(N, B, H, us, ds, seed=7), label=f"rows a few times apart, N={N}")


def _random_magnitude_cases(n, seed):
    rng = np.random.default_rng(seed)
    lengths = [256, 512, 1024, 2048, 4096, 8192, 16384, 32768, 65536]
    p = np.array([4, 4, 4, 4, 3, 3, 2, 1, 1], dtype=float)
    cases = []
    for _ in range(n):
        N = int(rng.choice(lengths, p=p / p.sum()))
        B = int(rng.integers(1, 12)) if N <= 4096 else int(rng.integers(1, 5))
        H = int(rng.integers(1, 7)) if N <= 16384 else int(rng.integers(1, 3))
        cases.append((N, B, H, int(rng.integers(0, 10000)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("N,B,H,seed,kernels", _random_magnitude_cases(48, 20230213))
def test_random_magnitudes(N, B, H, seed, kernels):
    # rows at 10^-6 ... 10^6 (u) and 10^-9 ... 10^3 (dy), drawn row by row up to N = 16384 and head by head beyond (the
    # multi-pass plans scale per head), kernels and skip terms at 2^-24 ... 2^20 in half of the cases: y, du and dk to
    # the bound of data of order one, every row and head.  dD is a plain fp32 dot product over all rows of a head:
    # where rows of wildly different size meet in one sum its relative error reaches a few 1e-5 (1e-7 otherwise).
    rng = np.random.default_rng(seed)
    shape = (B, H) if N <= 16384 else (1, H)
    us = np.broadcast_to(10.0 ** rng.uniform(-6, 6, size=shape), (B, H)).copy()
    ds = np.broadcast_to(10.0 ** rng.uniform(-9, 3, size=shape), (B, H)).copy()
    ks = 2.0 ** rng.integers(-24, 20, size=H) if kernels else None
    Ds = 2.0 ** rng.integers(-24, 20, size=H) if kernels else None
    check_full(scaled_inputs(N, B, H, us, ds, k_scale=ks, D_scale=Ds, seed=seed), label=f"random magnitudes, N={N}", dd_tol=1e-4)
