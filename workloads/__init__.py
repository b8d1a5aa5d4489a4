"""Seeded synthetic inputs for the long-convolution workloads.

This module serves both the CPU oracle and the GPU library and therefore holds
none of the convolution's arithmetic: it only draws random tensors, shapes the
synthetic kernels, and rounds tensors to the I/O precision.  Everything is
numpy on the host.

Workloads (shapes follow the regimes the paper trains in: language-model width
H=768, sequence lengths 1K..16K of its long-range benchmarks, 64K of its
longest task, kernels with exponential decay as in its geometric
initialisation, and soft-thresholded / smoothed kernels as its Squash and
Smooth regularisers of Section 3.1 produce):

  1  B=2,  H=4,    N=1024,            fp32   k = g*exp(-t/256),       g~N(0,1)
  2  B=16, H=768,  N=1024,            bf16   k = pool3(squash(g, .003)), g~N(0,0.02^2)
  3  B=8,  H=256,  N=16384,           fp16   k = squash(g*exp(-a_h t/N), 1e-4), g~N(0,1/N), a_h~U(.5,8)
  4  B=1,  H=128,  N=65536 | 131072,  fp16   k = g*exp(-4t/N),        g~N(0,1/N)
  5  B=64, H=1024, N in {256,512,2048,4096}, bf16   k as workload 2

u, D, dy ~ N(0,1) always.  N(0,x) means variance x.  The order "squash, then
pool" follows the workload definition (the paper's Algorithm 1 applies Smooth
before Squash); the pooling window is centred, three taps, zero padded at both
ends and always divided by three (the paper's Smooth formula is off-centre by
one and states no boundary rule).  These choices shape the synthetic kernel
only; both the oracle and the GPU consume the same generated tensors.

Seeding: numpy default_rng(20230213*10 + workload id [+ 1000*N for sweeps]),
child streams spawned in the fixed order u, g, alpha, D, dy.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F32, F16, BF16 = 0, 1, 2          # same integer codes as the C-ABI dtype enum
DTYPE_NAMES = {F32: "fp32", F16: "fp16", BF16: "bf16"}
DTYPE_BYTES = {F32: 4, F16: 2, BF16: 2}


@dataclass(frozen=True)
class Workload:
    wid: int
    B: int
    H: int
    N: int
    dtype: int
    kernel: str        # "decay256" | "squash_pool" | "decay_alpha_squash" | "decay4"

    @property
    def name(self) -> str:
        return f"cfg{self.wid}_B{self.B}_H{self.H}_N{self.N}_{DTYPE_NAMES[self.dtype]}"


WORKLOADS = {
    "1": Workload(1, 2, 4, 1024, F32, "decay256"),
    "2": Workload(2, 16, 768, 1024, BF16, "squash_pool"),
    "3": Workload(3, 8, 256, 16384, F16, "decay_alpha_squash"),
    "4a": Workload(4, 1, 128, 65536, F16, "decay4"),
    "4b": Workload(4, 1, 128, 131072, F16, "decay4"),
    "5_256": Workload(5, 64, 1024, 256, BF16, "squash_pool"),
    "5_512": Workload(5, 64, 1024, 512, BF16, "squash_pool"),
    "5_2048": Workload(5, 64, 1024, 2048, BF16, "squash_pool"),
    "5_4096": Workload(5, 64, 1024, 4096, BF16, "squash_pool"),
}


# ----------------------------------------------------------------------------
# rounding to the I/O precision (round-to-nearest-even), bit patterns for upload
# ----------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: int):
    """Round float32 `x` to the I/O dtype.

    Returns (storage, values): `storage` is what is uploaded to the GPU
    (float32 array, float16 array, or uint16 bf16 bit patterns) and `values`
    is the same numbers as float64, which is what the oracle consumes.
    """
    x = np.asarray(x, dtype=np.float32)
    if dtype == F32:
        return x, x.astype(np.float64)
    if dtype == F16:
        s = x.astype(np.float16)
        return s, s.astype(np.float64)
    if dtype == BF16:
        s = bf16_bits(x)
        return s, bf16_to_f32(s).astype(np.float64)
    raise ValueError(f"bad dtype {dtype}")


def storage_to_f64(storage: np.ndarray, dtype: int) -> np.ndarray:
    """Inverse view of quantize(): GPU output storage -> float64 values."""
    if dtype == BF16:
        return bf16_to_f32(np.asarray(storage, dtype=np.uint16)).astype(np.float64)
    return np.asarray(storage).astype(np.float64)


# ----------------------------------------------------------------------------
# synthetic kernel shaping (generator side of the paper's Section 3.1 operators)
# ----------------------------------------------------------------------------
def squash(k: np.ndarray, lam: float) -> np.ndarray:
    """Soft threshold sign(k)*max(|k|-lam, 0) (the paper's Squash operator)."""
    return (np.sign(k) * np.maximum(np.abs(k) - lam, 0.0)).astype(k.dtype)


def pool3(k: np.ndarray) -> np.ndarray:
    """Centred 3-tap average along the last axis, zero padded, always /3."""
    p = np.zeros(k.shape[:-1] + (k.shape[-1] + 2,), dtype=k.dtype)
    p[..., 1:-1] = k
    return ((p[..., :-2] + p[..., 1:-1] + p[..., 2:]) / 3.0).astype(k.dtype)


def make_kernel(kind: str, H: int, N: int, rng_g, rng_a) -> np.ndarray:
    t = np.arange(N, dtype=np.float64)[None, :]
    if kind == "decay256":
        g = rng_g.standard_normal((H, N))
        k = g * np.exp(-t / 256.0)
    elif kind == "squash_pool":
        g = 0.02 * rng_g.standard_normal((H, N))
        k = pool3(squash(g, 0.003))
    elif kind == "decay_alpha_squash":
        g = rng_g.standard_normal((H, N)) / np.sqrt(N)
        a = rng_a.uniform(0.5, 8.0, size=(H, 1))
        k = squash(g * np.exp(-a * t / N), 1e-4)
    elif kind == "decay4":
        g = rng_g.standard_normal((H, N)) / np.sqrt(N)
        k = g * np.exp(-4.0 * t / N)
    else:
        raise ValueError(kind)
    return k.astype(np.float32)


@dataclass
class Inputs:
    """One seeded input set. *_store is the upload form, the float64 fields feed the oracle."""
    w: Workload
    u_store: np.ndarray
    dy_store: np.ndarray
    u: np.ndarray
    dy: np.ndarray
    k: np.ndarray      # float32 [H,N] (library input; oracle upcasts)
    D: np.ndarray      # float32 [H]


def generate(w: Workload, *, B: int | None = None, H: int | None = None, seed_extra: int = 0) -> Inputs:
    """Draw the seeded tensors of workload `w` (optionally with B or H overridden for small cases)."""
    B = w.B if B is None else B
    H = w.H if H is None else H
    seed = 20230213 * 10 + w.wid + (1000 * w.N if w.wid == 5 else 0) + seed_extra
    r_u, r_g, r_a, r_D, r_dy = np.random.default_rng(seed).spawn(5)
    u32 = r_u.standard_normal((B, H, w.N), dtype=np.float32)
    k = make_kernel(w.kernel, H, w.N, r_g, r_a)
    D = r_D.standard_normal(H).astype(np.float32)
    dy32 = r_dy.standard_normal((B, H, w.N), dtype=np.float32)
    u_s, u_v = quantize(u32, w.dtype)
    dy_s, dy_v = quantize(dy32, w.dtype)
    return Inputs(w, u_s, dy_s, u_v, dy_v, k, D)


# ----------------------------------------------------------------------------
# byte / flop models used by the benchmark (user-visible tensors only)
# ----------------------------------------------------------------------------
def algorithmic_bytes(B: int, H: int, N: int, dtype: int):
    """(fwd bytes, bwd bytes): u,y,dy,du in the I/O dtype; k,D,dk,dD in fp32."""
    s = DTYPE_BYTES[dtype]
    E = B * H * N
    return 2 * E * s + H * N * 4 + H * 4, 3 * E * s + 2 * H * N * 4 + 2 * H * 4


def algorithmic_flops(B: int, H: int, N: int):
    """(fwd flops, bwd flops) from the standard real-FFT count 2.5*L*log2(L), L=2N."""
    lg = np.log2(2 * N)
    rows = B * H
    return rows * (10 * N * lg + 8 * N), rows * (15 * N * lg + 18 * N) + H * 5 * N * lg


def rel_l2(x, ref) -> float:
    """||x-ref||_2 / ||ref||_2 over the whole tensor, in float64."""
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / den) if den > 0 else float(np.linalg.norm(x - ref))
