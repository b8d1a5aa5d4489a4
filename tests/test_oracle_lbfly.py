"""Pins of the learned-Butterfly oracle against things it does not compute itself."""
import numpy as np
import pytest

import oracle
from oracle import lbfly


def _rand_blocks(H, L, seed, eps=0.3):
    """DFT blocks plus a complex perturbation of relative size eps."""
    Af, Ai = lbfly.dft_blocks(H, L)
    rng = np.random.default_rng(seed)
    pert = lambda: eps * (rng.standard_normal(Af.shape) + 1j * rng.standard_normal(Af.shape))
    return Af + pert(), Ai + pert()


def _problem(B, H, N, seed):
    rng = np.random.default_rng(seed)
    u, dy = rng.standard_normal((B, H, N)), rng.standard_normal((B, H, N))
    k, D = rng.standard_normal((H, N)) / np.sqrt(N), rng.standard_normal(H)
    return u, dy, k, D


@pytest.mark.parametrize("N", [16, 64, 256, 1024])
def test_dft_blocks_give_the_causal_convolution_and_its_gradients(N):
    B, H = 2, 2
    u, dy, k, D = _problem(B, H, N, 1)
    Af, Ai = lbfly.dft_blocks(H, 2 * N)
    shat = lbfly.spectrum(k, D)
    y = lbfly.lbfly_fwd(u, shat, Af, Ai)
    assert np.allclose(y, oracle.longconv_fwd(u, k, D), rtol=1e-10, atol=1e-10)
    du, dshat, _, _ = lbfly.lbfly_bwd(dy, u, shat, Af, Ai)
    dk, dD = lbfly.spectrum_bwd(dshat, N)
    rdu, rdk, rdD = oracle.longconv_bwd(dy, u, k, D)
    assert np.allclose(du, rdu, rtol=1e-10, atol=1e-10)
    assert np.allclose(dk, rdk, rtol=1e-10, atol=1e-10) and np.allclose(dD, rdD, rtol=1e-10, atol=1e-10)


@pytest.mark.parametrize("L", [32, 128, 512])
def test_stage_chain_equals_the_dense_kronecker_product(L):
    # every stage as an explicit L x L matrix, kron(I, kron(A_s, I_{M_s})), and every twiddle as a diagonal:
    # T_A = prod_s D_s (I (x) A_s (x) I); with DFT blocks that matrix is the DFT up to the digit-reversed order
    r, M = lbfly.stages(L)
    S = len(r)
    Af, Ai = _rand_blocks(1, L, 2)
    tw, freq = lbfly.twiddles(L)

    def dense(blocks, inverse):
        T = np.eye(L, dtype=np.complex128)
        order = range(S - 1, -1, -1) if inverse else range(S)
        for s in order:
            stage = np.kron(np.eye(L // (r[s] * M[s])), np.kron(blocks[0, s, :r[s], :r[s]], np.eye(M[s])))
            d = np.diag(tw[s].reshape(-1)) if s < S - 1 else np.eye(L)
            T = (stage @ np.conj(d) @ T) if inverse else (d @ stage @ T)
        return T

    TA, TB = dense(Af, False), dense(Ai, True)
    rng = np.random.default_rng(3)
    N = L // 2
    u = rng.standard_normal((1, 1, N))
    shat = (rng.standard_normal((1, L)) + 1j * rng.standard_normal((1, L)))
    x = np.concatenate([u[0, 0], np.zeros(N)])
    ref = np.real(TB @ (shat[0][freq.reshape(-1)] * (TA @ x)))[:N] / L
    assert np.allclose(lbfly.lbfly_fwd(u, shat, Af, Ai)[0, 0], ref, rtol=1e-11, atol=1e-11)
    F, Fi = lbfly.dft_blocks(1, L)
    Fm = dense(F, False)
    full = np.fft.fft(np.eye(L), axis=0)
    assert np.allclose(Fm, full[freq.reshape(-1), :], atol=1e-10)          # position p holds frequency freq[p]
    assert np.allclose(dense(Fi, True) @ Fm / L, np.eye(L), atol=1e-10)


def test_bilinearity_identities_hold_for_every_argument():
    B, H, N = 3, 2, 64
    u, dy, k, D = _problem(B, H, N, 4)
    Af, Ai = _rand_blocks(H, 2 * N, 5)
    shat = lbfly.spectrum(k, D)
    loss = np.sum(dy * lbfly.lbfly_fwd(u, shat, Af, Ai))
    du, dshat, dAf, dAi = lbfly.lbfly_bwd(dy, u, shat, Af, Ai)
    assert np.isclose(np.sum(du * u), loss, rtol=1e-11)
    assert np.isclose(np.real(np.sum(np.conj(dshat) * shat)), loss, rtol=1e-11)
    for s in range(Af.shape[1]):        # y is linear in every block separately
        assert np.isclose(np.real(np.sum(np.conj(dAf[:, s]) * Af[:, s])), loss, rtol=1e-11)
        assert np.isclose(np.real(np.sum(np.conj(dAi[:, s]) * Ai[:, s])), loss, rtol=1e-11)


@pytest.mark.parametrize("N", [16, 128])
def test_central_differences_in_every_argument(N):
    B, H = 2, 2
    u, dy, k, D = _problem(B, H, N, 6)
    Af, Ai = _rand_blocks(H, 2 * N, 7)
    shat = lbfly.spectrum(k, D)
    du, dshat, dAf, dAi = lbfly.lbfly_bwd(dy, u, shat, Af, Ai)
    args = {"u": u, "shat": shat, "Af": Af, "Ai": Ai}
    grads = {"u": du, "shat": dshat, "Af": dAf, "Ai": dAi}
    f = lambda a: np.sum(dy * lbfly.lbfly_fwd(a["u"], a["shat"], a["Af"], a["Ai"]))
    rng = np.random.default_rng(8)
    r, _ = lbfly.stages(2 * N)
    eps = 1e-6
    for name in args:
        for _ in range(8):
            idx = tuple(int(rng.integers(0, s)) for s in args[name].shape)
            if name in ("Af", "Ai"):
                rs = r[idx[1]]
                idx = (idx[0], idx[1], idx[2] % rs, idx[3] % rs)
            for part in ((1.0,) if name == "u" else (1.0, 1j)):
                hi, lo = dict(args), dict(args)
                hi[name], lo[name] = args[name].copy(), args[name].copy()
                hi[name][idx] += eps * part
                lo[name][idx] -= eps * part
                fd = (f(hi) - f(lo)) / (2 * eps)
                g = grads[name][idx]
                want = np.real(g) if part == 1.0 else np.imag(g)
                assert np.isclose(fd, want, rtol=1e-6, atol=1e-8), (name, idx, part)


def test_entries_outside_the_last_stage_corner_are_ignored():
    B, H, N = 1, 1, 16                      # L = 32: stages 16 and 2
    u, dy, k, D = _problem(B, H, N, 9)
    Af, Ai = _rand_blocks(H, 2 * N, 10)
    shat = lbfly.spectrum(k, D)
    y = lbfly.lbfly_fwd(u, shat, Af, Ai)
    Af2 = Af.copy()
    Af2[:, 1, 2:, :] = 7.0
    Af2[:, 1, :, 2:] = 7.0
    assert np.array_equal(y, lbfly.lbfly_fwd(u, shat, Af2, Ai))
    dAf = lbfly.lbfly_bwd(dy, u, shat, Af2, Ai)[2]
    assert np.all(dAf[:, 1, 2:, :] == 0) and np.all(dAf[:, 1, :, 2:] == 0)


def test_spectrum_and_its_adjoint():
    H, N = 2, 32
    rng = np.random.default_rng(11)
    k, D = rng.standard_normal((H, N)), rng.standard_normal(H)
    shat = lbfly.spectrum(k, D)
    L = 2 * N
    f, s = np.arange(L)[:, None], np.arange(N)[None, :]
    W = np.exp(-2j * np.pi * f * s / L)                       # the definition, written out
    assert np.allclose(shat, (W @ k.T).T + D[:, None])
    g = rng.standard_normal((H, L)) + 1j * rng.standard_normal((H, L))
    dk, dD = lbfly.spectrum_bwd(g, N)
    assert np.isclose(np.sum(dk * k) + np.sum(dD * D), np.real(np.sum(np.conj(g) * shat)), rtol=1e-12)
