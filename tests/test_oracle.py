"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test is chosen so that a plausible mistake in oracle.c (dropped D term,
wrong sign or index base, wrap-around, transposed operand in an adjoint) fails
at least one of them.
"""
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(7)


def _rand(B, H, N):
    return (RNG.standard_normal((B, H, N)), RNG.standard_normal((H, N)), RNG.standard_normal(H))


def test_hand_worked_example_eq1():
    vals = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_worked_example.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, *nums = line.split()
        vals[name] = np.array([float(x) for x in nums])
    u = vals["u"].reshape(1, 1, 4); k = vals["k"].reshape(1, 4); D = vals["D"]
    dy = vals["dy"].reshape(1, 1, 4)
    assert np.array_equal(oracle.longconv_fwd(u, k, D).ravel(), vals["y"])
    du, dk, dD = oracle.longconv_bwd(dy, u, k, D)
    assert np.array_equal(du.ravel(), vals["du"])
    assert np.array_equal(dk.ravel(), vals["dk"])
    assert np.array_equal(dD, vals["dD"])


def test_delta_kernel_returns_u_and_skip_adds():
    u, k, D = _rand(3, 2, 64)
    k[:] = 0.0; k[:, 0] = 1.0
    assert np.array_equal(oracle.longconv_fwd(u, k, 0 * D), u)
    y = oracle.longconv_fwd(u, k, D)
    np.testing.assert_allclose(y, (1.0 + D)[None, :, None] * u, rtol=1e-15, atol=0)


@pytest.mark.parametrize("shift", [1, 5, 63])
def test_shifted_delta_shifts_without_wraparound(shift):
    u, k, D = _rand(2, 3, 64)
    k[:] = 0.0; k[:, shift] = 1.0
    y = oracle.longconv_fwd(u, k, 0 * D)
    assert np.array_equal(y[..., shift:], u[..., : 64 - shift])
    assert np.all(y[..., :shift] == 0.0)          # causal: nothing wraps to the front


def test_bilinearity():
    u1, k1, D1 = _rand(2, 3, 96)
    u2, k2, D2 = _rand(2, 3, 96)
    a, b = 0.7, -1.3
    f = oracle.longconv_fwd
    np.testing.assert_allclose(f(a * u1 + b * u2, k1, D1), a * f(u1, k1, D1) + b * f(u2, k1, D1), atol=1e-12)
    np.testing.assert_allclose(f(u1, a * k1 + b * k2, a * D1 + b * D2),
                               a * f(u1, k1, D1) + b * f(u1, k2, D2), atol=1e-12)
    # D term is additive and separate from the convolution term
    np.testing.assert_allclose(f(u1, k1, D1) - f(u1, k1, 0 * D1), D1[None, :, None] * u1, atol=1e-12)


def test_all_ones_kernel_is_prefix_sum():
    u, k, D = _rand(2, 2, 200)
    k[:] = 1.0
    np.testing.assert_allclose(oracle.longconv_fwd(u, k, 0 * D), np.cumsum(u, axis=-1), atol=1e-12)


def test_geometric_kernel_is_first_order_recurrence():
    # One-state SSM of Section 2: x_t = a x_{t-1} + u_t, y_t = x_t + D u_t  <=>  k[t] = a^t.
    u, k, D = _rand(2, 3, 128)
    a = np.array([0.9, -0.5, 0.99])
    k[:] = a[:, None] ** np.arange(128)[None, :]
    y = oracle.longconv_fwd(u, k, D)
    x = np.zeros((2, 3)); ref = np.empty_like(u)
    for t in range(128):
        x = a[None, :] * x + u[..., t]
        ref[..., t] = x + D[None, :] * u[..., t]
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def _dft_matrix(L):
    n = np.arange(L)
    return np.exp(-2j * np.pi * np.outer(n, n) / L)


@pytest.mark.parametrize("N", [4, 16, 64])
def test_brute_force_dft_route_eq2(N):
    # Eq. 2 route written out with an explicit O(L^2) DFT matrix, zero padded to 2N.
    u, k, D = _rand(2, 2, N)
    L = 2 * N
    F = _dft_matrix(L); Finv = np.conj(F) / L
    up = np.concatenate([u, np.zeros_like(u)], -1); kp = np.concatenate([k, np.zeros_like(k)], -1)
    y_fft = np.einsum("ts,bhs->bht", Finv, np.einsum("fs,bhs->bhf", F, up) * (F @ kp.T).T[None])
    ref = y_fft.real[..., :N] + D[None, :, None] * u
    y = oracle.longconv_fwd(u, k, D)
    np.testing.assert_allclose(y, ref, atol=1e-11)
    # the unpadded (circular) reading of Eq. 2 is a different function
    Fn = _dft_matrix(N)
    circ = (np.conj(Fn) / N @ ((Fn @ u[0, 0]) * (Fn @ k[0]))).real + D[0] * u[0, 0]
    assert np.abs(circ - y[0, 0]).max() > 1e-3


def test_matches_numpy_convolve():
    u, k, D = _rand(3, 4, 257)
    ref = np.stack([[np.convolve(u[b, h], k[h])[:257] + D[h] * u[b, h] for h in range(4)] for b in range(3)])
    np.testing.assert_allclose(oracle.longconv_fwd(u, k, D), ref, atol=1e-12)


def test_backward_adjoint_identities():
    B, H, N = 3, 4, 80
    u, k, D = _rand(B, H, N)
    dy = RNG.standard_normal((B, H, N)); v = RNG.standard_normal((B, H, N))
    w = RNG.standard_normal((H, N)); e = RNG.standard_normal(H)
    du, dk, dD = oracle.longconv_bwd(dy, u, k, D)
    f = oracle.longconv_fwd
    # <dy, f(v;k,D)> = <du, v>
    np.testing.assert_allclose(np.vdot(dy, f(v, k, D)), np.vdot(du, v), rtol=1e-12)
    # <dy, f(u;w,0)> = <dk, w>,  <dy, f(u;0,e)> = <dD, e>
    np.testing.assert_allclose(np.vdot(dy, f(u, w, 0 * e)), np.vdot(dk, w), rtol=1e-12)
    np.testing.assert_allclose(np.vdot(dy, f(u, 0 * w, e)), np.vdot(dD, e), rtol=1e-12)
    np.testing.assert_allclose(dD, np.einsum("bht,bht->h", dy, u), rtol=1e-12)


def test_backward_flip_identities():
    B, H, N = 2, 3, 70
    u, k, D = _rand(B, H, N)
    dy = RNG.standard_normal((B, H, N))
    du, dk, _ = oracle.longconv_bwd(dy, u, k, D)
    z = np.zeros(H)
    du_ref = oracle.longconv_fwd(dy[..., ::-1], k, z)[..., ::-1] + D[None, :, None] * dy
    np.testing.assert_allclose(du, du_ref, atol=1e-12)
    dk_ref = np.zeros((H, N))
    for b in range(B):
        for h in range(H):
            dk_ref[h] += np.convolve(dy[b, h, ::-1], u[b, h])[:N][::-1]
    np.testing.assert_allclose(dk, dk_ref, atol=1e-12)


def test_backward_finite_differences():
    B, H, N = 2, 2, 24
    u, k, D = _rand(B, H, N)
    dy = RNG.standard_normal((B, H, N))
    du, dk, dD = oracle.longconv_bwd(dy, u, k, D)
    loss = lambda uu, kk, DD: float(np.vdot(dy, oracle.longconv_fwd(uu, kk, DD)))
    eps = 1e-3   # bilinear map: central differences are exact up to rounding
    for idx in [(0, 0, 0), (1, 1, 7), (0, 1, N - 1)]:
        e = np.zeros_like(u); e[idx] = eps
        np.testing.assert_allclose((loss(u + e, k, D) - loss(u - e, k, D)) / (2 * eps), du[idx], rtol=1e-8)
    for idx in [(0, 0), (1, 5), (1, N - 1)]:
        e = np.zeros_like(k); e[idx] = eps
        np.testing.assert_allclose((loss(u, k + e, D) - loss(u, k - e, D)) / (2 * eps), dk[idx], rtol=1e-8)
    for h in range(H):
        e = np.zeros_like(D); e[h] = eps
        np.testing.assert_allclose((loss(u, k, D + e) - loss(u, k, D - e)) / (2 * eps), dD[h], rtol=1e-8)


def test_row_and_head_subsets_are_independent():
    B, H, N = 3, 4, 50
    u, k, D = _rand(B, H, N)
    dy = RNG.standard_normal((B, H, N))
    y = oracle.longconv_fwd(u, k, D)
    du, dk, dD = oracle.longconv_bwd(dy, u, k, D)
    hs = [1, 3]
    np.testing.assert_array_equal(oracle.longconv_fwd(u[:, hs], k[hs], D[hs]), y[:, hs])
    np.testing.assert_array_equal(oracle.longconv_bwd_du(dy[1:2, hs], k[hs], D[hs]), du[1:2, hs])
    dk2, dD2 = oracle.longconv_bwd_dk_dD(dy[:, hs], u[:, hs])
    np.testing.assert_array_equal(dk2, dk[hs]); np.testing.assert_array_equal(dD2, dD[hs])
