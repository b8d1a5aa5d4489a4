"""Pins of the gated-convolution oracle: things the product rule and Eq. 1 fix without calling the oracle's own
formulas again."""
import numpy as np

import oracle
from oracle import gated


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_unit_gate_is_the_ungated_layer():
    B, H, N = 2, 3, 16
    u, k, D, dy = _rand((B, H, N), 0), _rand((H, N), 1), _rand(H, 2), _rand((B, H, N), 3)
    one = np.ones((B, H, N))
    assert np.array_equal(gated.gated_fwd(u, k, D, one), oracle.longconv_fwd(u, k, D))
    du, dk, dD, dg = gated.gated_bwd(dy, one, u, k, D)
    rdu, rdk, rdD = oracle.longconv_bwd(dy, u, k, D)
    assert np.array_equal(du, rdu) and np.array_equal(dk, rdk) and np.array_equal(dD, rdD)
    assert np.array_equal(dg, dy * oracle.longconv_fwd(u, k, D))


def test_one_hot_gate_picks_one_output_sample_worked_by_hand():
    # N = 4, one row: z = (k*u)[:4] + D u with k = (1, 2, 0, -1), u = (3, -1, 2, 1), D = 0.5
    # z0 = 3 + 1.5 = 4.5; z1 = -1 + 6 - 0.5 = 4.5; z2 = 2 - 2 + 0 + 1 = 1; z3 = 1 + 4 + 0 - 3 + 0.5 = 2.5
    u = np.array([[[3.0, -1.0, 2.0, 1.0]]])
    k = np.array([[1.0, 2.0, 0.0, -1.0]])
    D = np.array([0.5])
    g = np.array([[[0.0, 0.0, 2.0, 0.0]]])
    assert np.allclose(gated.gated_fwd(u, k, D, g), [[[0.0, 0.0, 2.0, 0.0]]])
    g2 = np.array([[[1.0, -1.0, 0.0, 4.0]]])
    assert np.allclose(gated.gated_fwd(u, k, D, g2), [[[4.5, -4.5, 0.0, 10.0]]])
    # backward with dy = (0,0,1,0), g = (0,0,2,0): dz = (0,0,2,0)
    # du[s] = sum_{t>=s} k[t-s] dz[t] + D dz[s] = 2 k[2-s] (s<=2) + (s==2) -> (0, 4, 2 + 1, 0)
    # dk[s] = sum_{t>=s} dz[t] u[t-s] = 2 u[2-s] (s<=2) -> (4, -2, 6, 0); dD = 2 u[2] = 4; dg = dy * z = (0,0,1,0)
    dy = np.array([[[0.0, 0.0, 1.0, 0.0]]])
    du, dk, dD, dg = gated.gated_bwd(dy, g, u, k, D)
    assert np.allclose(du, [[[0.0, 4.0, 3.0, 0.0]]])
    assert np.allclose(dk, [[4.0, -2.0, 6.0, 0.0]])
    assert np.allclose(dD, [4.0])
    assert np.allclose(dg, [[[0.0, 0.0, 1.0, 0.0]]])


def test_bilinearity_identities():
    # L = <dy, y> is linear in g and in u (k, D fixed): <dg, g> = L = <du, u>; and linear in (k, D) jointly:
    # <dk, k> + <dD, D> = L
    B, H, N = 3, 2, 32
    u, k, D, g, dy = _rand((B, H, N), 4), _rand((H, N), 5), _rand(H, 6), _rand((B, H, N), 7), _rand((B, H, N), 8)
    L = np.sum(dy * gated.gated_fwd(u, k, D, g))
    du, dk, dD, dg = gated.gated_bwd(dy, g, u, k, D)
    assert np.isclose(np.sum(dg * g), L, rtol=1e-12)
    assert np.isclose(np.sum(du * u), L, rtol=1e-12)
    assert np.isclose(np.sum(dk * k) + np.sum(dD * D), L, rtol=1e-12)


def test_finite_differences_of_every_argument():
    B, H, N = 2, 2, 8
    u, k, D, g, dy = _rand((B, H, N), 9), _rand((H, N), 10), _rand(H, 11), _rand((B, H, N), 12), _rand((B, H, N), 13)
    du, dk, dD, dg = gated.gated_bwd(dy, g, u, k, D)

    def loss(u_, k_, D_, g_):
        return float(np.sum(dy * gated.gated_fwd(u_, k_, D_, g_)))

    eps = 1e-6
    rng = np.random.default_rng(14)
    for name, grad, arr in (("u", du, u), ("k", dk, k), ("D", dD, D), ("g", dg, g)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = {"u": u, "k": k, "D": D, "g": g}
            args_lo = dict(args_hi)
            args_hi[name], args_lo[name] = hi, lo
            fd = (loss(args_hi["u"], args_hi["k"], args_hi["D"], args_hi["g"]) -
                  loss(args_lo["u"], args_lo["k"], args_lo["D"], args_lo["g"])) / (2 * eps)
            assert np.isclose(fd, grad[idx], rtol=1e-6, atol=1e-8), (name, idx, fd, grad[idx])


def test_a_wrong_product_rule_would_be_caught():
    # dg must use the UNGATED output and dz must use g, not the other way round
    B, H, N = 1, 1, 8
    u, k, D, g, dy = _rand((B, H, N), 15), _rand((H, N), 16), _rand(H, 17), _rand((B, H, N), 18), _rand((B, H, N), 19)
    du, dk, dD, dg = gated.gated_bwd(dy, g, u, k, D)
    wrong_dg = dy * gated.gated_fwd(u, k, D, g)
    assert not np.allclose(dg, wrong_dg)
    wrong_du, _, _ = oracle.longconv_bwd(dy, u, k, D)
    assert not np.allclose(du, wrong_du)
