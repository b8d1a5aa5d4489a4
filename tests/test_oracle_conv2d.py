"""Pins of the 2-D convolution oracle against things it does not compute itself."""
import numpy as np
import scipy.signal

import oracle
from oracle import conv2d


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_against_scipy_full_convolution_truncated():
    B, H, N1, N2 = 2, 3, 5, 7
    u, k, D = _rand((B, H, N1, N2), 0), _rand((H, N1, N2), 1), _rand(H, 2)
    y = conv2d.conv2d_fwd(u, k, D)
    for b in range(B):
        for h in range(H):
            ref = scipy.signal.convolve2d(u[b, h], k[h], mode="full")[:N1, :N2] + D[h] * u[b, h]
            assert np.allclose(y[b, h], ref, rtol=1e-12, atol=1e-12)


def test_hand_worked_2x2():
    # u = [[1,2],[3,4]], k = [[1,-1],[2,0]], D = 0.5
    # y00 = 1*1 + .5 = 1.5; y01 = 1*2 - 1*1 + 1 = 2; y10 = 1*3 + 2*1 + 1.5 = 6.5; y11 = 4 - 3 + 2*2 + 0 + 2 = 7
    u = np.array([[[[1.0, 2.0], [3.0, 4.0]]]])
    k = np.array([[[1.0, -1.0], [2.0, 0.0]]])
    D = np.array([0.5])
    assert np.allclose(conv2d.conv2d_fwd(u, k, D), [[[[1.5, 2.0], [6.5, 7.0]]]])


def test_delta_filters_shift_the_image_and_nothing_wraps():
    B, H, N1, N2 = 1, 1, 4, 6
    u = _rand((B, H, N1, N2), 3)
    k = np.zeros((H, N1, N2))
    k[0, 1, 2] = 1.0
    y = conv2d.conv2d_fwd(u, k, np.zeros(H))
    ref = np.zeros_like(u)
    ref[:, :, 1:, 2:] = u[:, :, :-1, :-2]
    assert np.allclose(y, ref)


def test_separable_filter_is_two_1d_convolutions():
    # k[p,q] = a[p] b[q]: convolve every row with b (the 1-D oracle, rows as batch), then every column with a
    B, H, N1, N2 = 2, 2, 8, 8
    u, a, b = _rand((B, H, N1, N2), 4), _rand((H, N1), 5), _rand((H, N2), 6)
    k = a[:, :, None] * b[:, None, :]
    y = conv2d.conv2d_fwd(u, k, np.zeros(H))
    rows = np.stack([oracle.longconv_fwd(u[:, :, i, :], b, np.zeros(H)) for i in range(N1)], axis=2)
    cols = np.stack([oracle.longconv_fwd(rows[:, :, :, j], a, np.zeros(H)) for j in range(N2)], axis=3)
    assert np.allclose(y, cols, rtol=1e-11, atol=1e-11)


def test_adjoint_identities_and_finite_differences():
    B, H, N1, N2 = 2, 2, 4, 4
    u, k, D, dy = _rand((B, H, N1, N2), 7), _rand((H, N1, N2), 8), _rand(H, 9), _rand((B, H, N1, N2), 10)
    L = np.sum(dy * conv2d.conv2d_fwd(u, k, D))
    du, dk, dD = conv2d.conv2d_bwd(dy, u, k, D)
    assert np.isclose(np.sum(du * u), L, rtol=1e-12)
    assert np.isclose(np.sum(dk * k) + np.sum(dD * D), L, rtol=1e-12)
    eps = 1e-6
    rng = np.random.default_rng(11)
    for name, grad, arr in (("u", du, u), ("k", dk, k), ("D", dD, D)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = {"u": u, "k": k, "D": D}
            a_hi, a_lo = dict(args), dict(args)
            a_hi[name], a_lo[name] = hi, lo
            fd = (np.sum(dy * conv2d.conv2d_fwd(a_hi["u"], a_hi["k"], a_hi["D"])) -
                  np.sum(dy * conv2d.conv2d_fwd(a_lo["u"], a_lo["k"], a_lo["D"]))) / (2 * eps)
            assert np.isclose(fd, grad[idx], rtol=1e-6, atol=1e-8), (name, idx)


def test_row_padded_flattening_is_the_1d_convolution():
    # the identity the GPU path rests on: pad every row of image and filter to 2 N2, flatten row-major, convolve in
    # 1-D (causal, truncated), keep columns below N2
    B, H, N1, N2 = 2, 2, 4, 8
    u, k, D = _rand((B, H, N1, N2), 12), _rand((H, N1, N2), 13), _rand(H, 14)
    W = 2 * N2
    up = np.zeros((B, H, N1, W)); up[..., :N2] = u
    kp = np.zeros((H, N1, W)); kp[..., :N2] = k
    y1 = oracle.longconv_fwd(up.reshape(B, H, N1 * W), kp.reshape(H, N1 * W), D).reshape(B, H, N1, W)[..., :N2]
    assert np.allclose(y1, conv2d.conv2d_fwd(u, k, D), rtol=1e-11, atol=1e-11)
