"""CPU oracle for the kernel regularisers in front of the long convolution (float64, plain numpy).

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing on the product path imports it.

What it computes (paper Algorithm 1, lines 1-3, and Section 3.1 "Regularizing the Kernel"):

    K1 = dropout(K)                      line 1: K1 = M * K, the mask M (0 or 1/(1-q) per entry) is an input
    K2 = Smooth(K1)                      line 2: average pooling along the sequence
    Kbar = Squash(K2)                    line 3: sign(K2) * max(|K2| - lambda, 0), entry-wise

and the chain rule back through the three steps (the paper gives no backward): the gradient with
respect to K of a loss whose gradient with respect to Kbar is given.

Readings where the paper leaves room (both stated for the GPU side as well):
  * Smooth is printed as (2p+1)^-1 sum_{j=1..2p+1} K_{k+j-p}, a window k-p+1 .. k+p+1 that is off-centre by
    one, with no rule for the ends.  Read here as the centred window k-p .. k+p, entries outside 0..N-1
    taken as zero, always divided by 2p+1 (so p = 0 is the identity).  This is the same reading the
    synthetic-kernel generator uses for "pool width 3" (p = 1).
  * Squash's gradient at |K2| = lambda exactly (a kink) is taken as 0 (the subgradient the strict
    inequality |K2| > lambda selects).
"""
from __future__ import annotations

import numpy as np


def dropout(k, mask):
    """Algorithm 1 line 1 with the random mask passed in (None: no dropout)."""
    k = np.asarray(k, dtype=np.float64)
    return k if mask is None else k * np.asarray(mask, dtype=np.float64)


def smooth(k, p: int):
    """Algorithm 1 line 2 (Section 3.1, Smooth): centred window of 2p+1 taps, zeros outside, / (2p+1)."""
    k = np.asarray(k, dtype=np.float64)
    N = k.shape[-1]
    out = np.zeros_like(k)
    for n in range(N):                       # plain definition, one output at a time
        lo, hi = max(0, n - p), min(N - 1, n + p)
        out[..., n] = k[..., lo:hi + 1].sum(axis=-1) / (2 * p + 1)
    return out


def squash(k, lam: float):
    """Algorithm 1 line 3 (Section 3.1, Squash): sign(k) * max(|k| - lam, 0)."""
    k = np.asarray(k, dtype=np.float64)
    return np.sign(k) * np.maximum(np.abs(k) - lam, 0.0)


def kernel_reg_fwd(k, mask, p: int, lam: float):
    """Kbar = Squash(Smooth(dropout(K))), Algorithm 1 lines 1-3 in that order."""
    return squash(smooth(dropout(k, mask), p), lam)


def kernel_reg_bwd(k, mask, p: int, lam: float, dkbar):
    """dK given dKbar: back through Squash (gate |K2| > lam), Smooth (its transpose: the same centred
    zero-padded window, written out as a scatter) and dropout (the mask)."""
    k2 = smooth(dropout(k, mask), p)
    d2 = np.asarray(dkbar, dtype=np.float64) * (np.abs(k2) > lam)
    N = d2.shape[-1]
    d1 = np.zeros_like(d2)
    for n in range(N):                       # output n of Smooth read inputs lo..hi: scatter its gradient back
        lo, hi = max(0, n - p), min(N - 1, n + p)
        d1[..., lo:hi + 1] += d2[..., n:n + 1] / (2 * p + 1)
    return d1 if mask is None else d1 * np.asarray(mask, dtype=np.float64)
