"""CPU oracle for the gated long convolution (float64).

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing on the product path imports it.

The language-model experiments of the paper (Section 4.1, the H3-style layer: two sequence operators whose
outputs are multiplied together as a gating mechanism) use the long convolution with a multiplicative gate on its
output.  The paper gives no formula; the reading taken, with g a second sequence of the layer's shape:

    z[b,h,t] = sum_{s<=t} k[h,s] u[b,h,t-s] + D[h] u[b,h,t]          Eq. 1 / Algorithm 1 line 4 (ungated)
    y[b,h,t] = g[b,h,t] * z[b,h,t]

and its backward by the product and chain rules (dy = gradient with respect to y):

    dz = dy * g                 what the ungated backward receives: du, dk, dD = adjoints of Eq. 1 applied to dz
    dg = dy * z                 z recomputed from u, k, D

Each step is the plain definition; the convolution and its adjoints are the package's own direct sums.
"""
from __future__ import annotations

import numpy as np

from . import longconv_bwd, longconv_fwd


def gated_fwd(u, k, D, g):
    """y = g * (causal convolution of u with k, plus D u)."""
    return np.asarray(g, dtype=np.float64) * longconv_fwd(u, k, D)


def gated_bwd(dy, g, u, k, D):
    """(du, dk, dD, dg) of the gated forward."""
    dy = np.asarray(dy, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    du, dk, dD = longconv_bwd(dy * g, u, k, D)
    dg = dy * longconv_fwd(u, k, D)
    return du, dk, dD, dg
