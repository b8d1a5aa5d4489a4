"""CPU oracle for the 2-D long convolution (float64, direct sums).

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing on the product path imports it.

The image experiments of the paper (Section 4.1) replace the S4ND layers by "2D long convolution filters"; no
formula is given.  Reading taken, the 2-D counterpart of Eq. 1 / Algorithm 1 line 4: one filter k[h] of the size of
the image per head, linear (zero padded, not circular) convolution anchored at the origin and truncated to the
image, plus the skip term,

    y[b,h,i,j] = sum_{p<=i} sum_{q<=j} k[h,p,q] u[b,h,i-p,j-q] + D[h] u[b,h,i,j]       0 <= i < N1, 0 <= j < N2

and its exact adjoints

    du[b,h,i,j] = sum_{p} sum_{q} k[h,p,q] dy[b,h,i+p,j+q] + D[h] dy[b,h,i,j]
    dk[h,p,q]   = sum_b sum_{i>=p} sum_{j>=q} dy[b,h,i,j] u[b,h,i-p,j-q]
    dD[h]       = sum_b sum_i sum_j dy[b,h,i,j] u[b,h,i,j]

written out as loops over the filter taps (each tap is one shifted multiply-add over the image).
"""
from __future__ import annotations

import numpy as np


def conv2d_fwd(u, k, D):
    u = np.asarray(u, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    B, H, N1, N2 = u.shape
    y = D[None, :, None, None] * u
    for p in range(N1):
        for q in range(N2):
            y[:, :, p:, q:] += k[None, :, p, q, None, None] * u[:, :, :N1 - p, :N2 - q]
    return y


def conv2d_bwd(dy, u, k, D):
    dy = np.asarray(dy, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    B, H, N1, N2 = u.shape
    du = D[None, :, None, None] * dy
    dk = np.zeros((H, N1, N2))
    for p in range(N1):
        for q in range(N2):
            du[:, :, :N1 - p, :N2 - q] += k[None, :, p, q, None, None] * dy[:, :, p:, q:]
            dk[:, p, q] = np.einsum("bhij,bhij->h", dy[:, :, p:, q:], u[:, :, :N1 - p, :N2 - q])
    dD = np.einsum("bhij,bhij->h", dy, u)
    return du, dk, dD
