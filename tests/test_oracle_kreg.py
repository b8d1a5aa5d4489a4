"""Pins of the regulariser oracle (Algorithm 1 lines 1-3) against things other than itself (no GPU)."""
import numpy as np
import pytest

from oracle import kreg

RNG = np.random.default_rng(11)


def test_squash_is_the_l1_proximal_step_brute_force():
    # Section 3.1: Squash is one step of an L1 proximal operator.  Brute force on a grid: the minimiser of
    # lam |x| + (x - k)^2 / 2 is the soft threshold of k at lam (the explicit formula of the section)
    lam = 0.3
    xs = np.linspace(-3, 3, 600001)
    for k in (-2.0, -0.31, -0.3, -0.1, 0.0, 0.05, 0.3, 0.7, 2.5):
        best = xs[np.argmin(lam * np.abs(xs) + 0.5 * (xs - k) ** 2)]
        assert abs(best - kreg.squash(np.array([k]), lam)[0]) < 2e-5


def test_squash_closed_forms():
    k = np.array([-1.0, -0.2, -0.1, 0.0, 0.1, 0.2, 1.0])
    np.testing.assert_allclose(kreg.squash(k, 0.2), [-0.8, 0.0, 0.0, 0.0, 0.0, 0.0, 0.8], atol=1e-16)
    assert np.array_equal(kreg.squash(k, 0.0), k)                       # lam = 0 is the identity
    g = 0.02 * RNG.standard_normal(200000)
    s = kreg.squash(g, 0.003)
    assert np.all(np.abs(s) <= np.abs(g)) and np.all(s * g >= 0)        # shrinks towards zero, keeps the sign
    assert np.all((s == 0) == (np.abs(g) <= 0.003))


def test_smooth_hand_example_and_edges():
    k = np.array([[3.0, 6.0, 9.0, 12.0, 0.0, -3.0]])
    np.testing.assert_allclose(kreg.smooth(k, 1), [[3.0, 6.0, 9.0, 7.0, 3.0, -1.0]], atol=1e-15)
    np.testing.assert_allclose(kreg.smooth(k, 2), [[18 / 5, 30 / 5, 30 / 5, 24 / 5, 18 / 5, 9 / 5]], atol=1e-15)
    assert np.array_equal(kreg.smooth(k, 0), k)                         # p = 0 is the identity
    c = np.full((2, 40), 1.5)
    s = kreg.smooth(c, 3)
    np.testing.assert_allclose(s[:, 3:-3], 1.5, atol=1e-15)             # a constant stays constant inside
    np.testing.assert_allclose(s[:, 0], 1.5 * 4 / 7, atol=1e-15)        # four of seven taps exist at the ends
    np.testing.assert_allclose(s[:, -1], 1.5 * 4 / 7, atol=1e-15)


@pytest.mark.parametrize("p", [1, 2, 5])
def test_smooth_is_numpy_convolve_same(p):
    k = RNG.standard_normal(97)
    ref = np.convolve(k, np.ones(2 * p + 1) / (2 * p + 1), mode="same")
    np.testing.assert_allclose(kreg.smooth(k[None], p)[0], ref, atol=1e-14)
    # centred: a unit pulse spreads symmetrically (the printed formula, off-centre by one, would not)
    e = np.zeros((1, 21)); e[0, 10] = 1.0
    s = kreg.smooth(e, p)[0]
    assert np.array_equal(s, s[::-1]) and s[10 - p] > 0 and s[10 + p] > 0 and s[10 + p + 1] == 0


def test_order_of_the_three_steps():
    # dropout, then Smooth, then Squash (Algorithm 1 lines 1, 2, 3): the other orders give other results
    k = np.array([[0.0, 0.9, 0.0, 0.0, 0.5, 0.5, 0.5]])
    m = np.array([[1.0, 1.0, 1.0, 1.0, 2.0, 0.0, 2.0]])
    got = kreg.kernel_reg_fwd(k, m, 1, 0.25)
    want = kreg.squash(kreg.smooth(k * m, 1), 0.25)
    assert np.array_equal(got, want)
    assert not np.allclose(got, kreg.smooth(kreg.squash(k * m, 0.25), 1))
    assert not np.allclose(got, kreg.squash(kreg.smooth(k, 1), 0.25) * m)
    np.testing.assert_allclose(got[0, :3], [0.05, 0.05, 0.05], atol=1e-15)   # 0.9 / 3 - 0.25


@pytest.mark.parametrize("p,lam,with_mask", [(0, 0.0, False), (1, 0.003, True), (3, 0.01, True), (2, 0.0, False)])
def test_backward_is_the_transpose_of_the_jacobian(p, lam, with_mask):
    H, N = 3, 48
    k = 0.02 * RNG.standard_normal((H, N))
    mask = (RNG.random((H, N)) > 0.25) / 0.75 if with_mask else None
    g = RNG.standard_normal((H, N))
    dk = kreg.kernel_reg_bwd(k, mask, p, lam, g)
    # central differences entry by entry (the map is piecewise linear: exact away from the kinks)
    eps = 1e-7
    k2 = kreg.smooth(kreg.dropout(k, mask), p)
    assert np.min(np.abs(np.abs(k2) - lam)) > 10 * eps or lam == 0.0
    fd = np.zeros_like(k)
    for h in range(H):
        for n in range(N):
            kp = k.copy(); kp[h, n] += eps
            km = k.copy(); km[h, n] -= eps
            fd[h, n] = np.sum(g * (kreg.kernel_reg_fwd(kp, mask, p, lam) - kreg.kernel_reg_fwd(km, mask, p, lam))) / (2 * eps)
    np.testing.assert_allclose(dk, fd, atol=1e-7)
    # adjoint identity with a direction v: <g, J v> = <J^T g, v>
    v = RNG.standard_normal((H, N)) * 1e-9
    jv = kreg.kernel_reg_fwd(k + v, mask, p, lam) - kreg.kernel_reg_fwd(k, mask, p, lam)
    assert abs(np.sum(g * jv) - np.sum(dk * v)) < 1e-12


def test_backward_special_cases():
    k = RNG.standard_normal((2, 30))
    g = RNG.standard_normal((2, 30))
    assert np.array_equal(kreg.kernel_reg_bwd(k, None, 0, 0.0, g), g * (np.abs(k) > 0))     # identity map
    assert np.array_equal(kreg.kernel_reg_bwd(k, None, 0, 1e9, g), np.zeros_like(g))        # everything squashed
    m = (RNG.random((2, 30)) > 0.5) * 2.0
    np.testing.assert_array_equal(kreg.kernel_reg_bwd(k, m, 0, 0.0, g), g * m * (np.abs(k * m) > 0))
    # Smooth alone is symmetric: its transpose is itself
    np.testing.assert_allclose(kreg.kernel_reg_bwd(k, None, 2, 0.0, g), kreg.smooth(g, 2) * 1.0, atol=1e-14)
