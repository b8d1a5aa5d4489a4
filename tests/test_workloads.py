"""Input generators: rounding, kernel shaping, determinism (no GPU needed)."""
import math

import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.0e-39]        # ties and a subnormal
    bits = wl.bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(wl.bf16_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_squash_sparsity_closed_form():
    g = 0.02 * np.random.default_rng(1).standard_normal(400000)
    k = wl.squash(g, 0.003)
    frac0 = np.mean(k == 0.0)
    assert abs(frac0 - math.erf(0.003 / (0.02 * math.sqrt(2)))) < 3e-3
    nz = k != 0
    np.testing.assert_allclose(np.abs(k[nz]), np.abs(g[nz]) - 0.003, rtol=0, atol=1e-15)
    assert np.all(np.sign(k[nz]) == np.sign(g[nz]))


def test_pool3_centred_zero_padded():
    k = np.array([[3.0, 6.0, 9.0, 12.0]])
    np.testing.assert_allclose(wl.pool3(k), [[3.0, 6.0, 9.0, 7.0]])


def test_generate_is_seeded_and_quantised():
    w = wl.WORKLOADS["2"]
    a = wl.generate(w, B=2, H=3)
    b = wl.generate(w, B=2, H=3)
    assert np.array_equal(a.u_store, b.u_store) and np.array_equal(a.k, b.k)
    assert a.u_store.dtype == np.uint16 and a.u.dtype == np.float64
    assert np.array_equal(wl.storage_to_f64(a.u_store, w.dtype), a.u)
    assert a.k.dtype == np.float32 and a.k.shape == (3, 1024)
    c = wl.generate(wl.WORKLOADS["3"], B=1, H=2)
    assert c.u_store.dtype == np.float16
    # decay + squash leaves an (almost) zero tail for the fastest-decaying head
    assert np.mean(c.k == 0.0) > 0.005


def test_byte_model_matches_table():
    assert wl.algorithmic_bytes(8, 256, 16384, wl.F16) == (150995968, 234883072)
    assert wl.algorithmic_bytes(16, 768, 1024, wl.BF16) == (53480448, 81795072)
    assert wl.algorithmic_bytes(1, 128, 65536, wl.F16) == (67109376, 117441536)
