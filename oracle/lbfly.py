"""CPU oracle for the learned Butterfly extension (Section 3.3), float64 / complex128.

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing on the product path imports it.

The paper's extension keeps the FFT convolution of Eq. 2, written with the Butterfly decomposition of Section 3.2
(small dense blocks F_r interleaved with fixed twiddle diagonals and permutations, Appendix C.1), and learns the
values of the blocks instead of fixing them to the DFT; with block size r that adds O(H r^2) parameters.  The paper
gives no formula beyond that.  Reading taken here:

  * L = 2N = 2^LG points, S = ceil(LG / 4) stages.  Position p = (d_0, ..., d_{S-1}), d_0 most significant; digits
    d_0 .. d_{S-2} have 4 bits (radix 16), d_{S-1} the remaining LG - 4 (S-1) bits (radix r_last = 2 .. 16);
    M_s = stride of digit s.
  * forward transform T_A[h]: for s = 0 .. S-1 apply the head's block A_s[h] (r_s x r_s, complex) along digit s,
    then (s < S-1) multiply position p, whose digit s is now k_s, by w_s(p) = exp(-2 pi i k_s (p mod M_s) / (r_s M_s))
    (the twiddle M_{j,k} of Appendix C.1).  With A_s = DFT this is the decimation-in-frequency FFT, frequency
    f = k_0 + 16 k_1 + 256 k_2 ... at position (k_0, k_1, ...).
  * the stored spectrum Shat[h] = FFT_L([k[h], 0_N]) + D[h] (Algorithm 2 lines 1-2, the skip term as a constant
    spectrum) is NOT touched by the extension: only the transforms around it are learned.
  * inverse transform T_B[h]: the mirror image, s = S-1 .. 0: (s < S-1) multiply by conj(w_s), then apply B_s[h]
    along digit s; finally 1/L.  With B_s = conj(DFT) this is the inverse FFT.
  * y[b,h,t] = Re( T_B[h]( Shat[h] . T_A[h]( [u[b,h], 0_N] ) ) )[t],  0 <= t < N.

With DFT blocks the result is Eq. 1 exactly.  Gradients: reverse mode through the stages, written out; a complex
parameter's gradient is dL/dRe + i dL/dIm.  Blocks are passed as [H, S, 16, 16] complex arrays; the last stage
reads its leading r_last x r_last corner only (the rest gets zero gradient).
"""
from __future__ import annotations

import numpy as np


def stages(L: int):
    """Radices r_s and strides M_s of the S stages of an L-point transform."""
    LG = int(np.log2(L))
    assert 1 << LG == L and LG >= 5
    S = (LG + 3) // 4
    r = [16] * (S - 1) + [1 << (LG - 4 * (S - 1))]
    M = [L // int(np.prod(r[:s + 1])) for s in range(S)]
    return r, M


def twiddles(L: int):
    """w_s as arrays over the digit grid (shape r_0 x ... x r_{S-1}), s = 0 .. S-2, and the frequency of each
    position after the forward transform."""
    r, M = stages(L)
    p = np.arange(L).reshape(r)
    grids = np.indices(r)
    tw = [np.exp(-2j * np.pi * grids[s] * (p % M[s]) / (r[s] * M[s])) for s in range(len(r) - 1)]
    freq = sum(grids[s] * int(np.prod(r[:s])) for s in range(len(r)))
    return tw, freq


def dft_blocks(H: int, L: int):
    """The blocks that make the extension the plain FFT convolution: A_s = F_r, B_s = conj(F_r)."""
    r, _ = stages(L)
    Af = np.zeros((H, len(r), 16, 16), dtype=np.complex128)
    for s, rs in enumerate(r):
        jk = np.outer(np.arange(rs), np.arange(rs))
        Af[:, s, :rs, :rs] = np.exp(-2j * np.pi * jk / rs)
    return Af, np.conj(Af)


def spectrum(k, D):
    """Shat[h] = FFT_L([k[h], 0_N]) + D[h]  (natural frequency order)."""
    k = np.asarray(k, dtype=np.float64)
    H, N = k.shape
    return np.fft.fft(np.concatenate([k, np.zeros_like(k)], axis=1), axis=1) + np.asarray(D, dtype=np.float64)[:, None]


def spectrum_bwd(dshat, N: int):
    """dk[h,s] = Re sum_f conj(exp(-2 pi i f s / L)) dShat[h,f] for s < N;  dD[h] = Re sum_f dShat[h,f]."""
    dshat = np.asarray(dshat, dtype=np.complex128)
    L = dshat.shape[1]
    dk = np.real(np.fft.ifft(dshat, axis=1) * L)[:, :N]
    return dk, np.real(dshat.sum(axis=1))


def _apply(mat, x, axis):
    """mat (r x r) along axis `axis` of x."""
    return np.moveaxis(np.tensordot(mat, x, axes=([1], [axis])), 0, axis)


def _outer(g, x, axis):
    """sum over every axis but `axis` of g (x) conj(x): an r x r matrix."""
    r = g.shape[axis]
    return np.moveaxis(g, axis, 0).reshape(r, -1) @ np.conj(np.moveaxis(x, axis, 0).reshape(r, -1)).T


def _forward_chain(x, A, tw, r):
    """T_A of one head on x [B, r_0, ..., r_{S-1}]; returns the inputs of every stage and the result."""
    xs = []
    for s, rs in enumerate(r):
        xs.append(x)
        x = _apply(A[s, :rs, :rs], x, 1 + s)
        if s < len(r) - 1:
            x = x * tw[s]
    return xs, x


def _inverse_chain(v, Bm, tw, r):
    ins = [None] * len(r)
    for s in range(len(r) - 1, -1, -1):
        if s < len(r) - 1:
            v = v * np.conj(tw[s])
        ins[s] = v
        v = _apply(Bm[s, :r[s], :r[s]], v, 1 + s)
    return ins, v


def lbfly_fwd(u, shat, Af, Ai):
    u = np.asarray(u, dtype=np.float64)
    B, H, N = u.shape
    L = 2 * N
    r, _ = stages(L)
    tw, freq = twiddles(L)
    y = np.empty_like(u)
    for h in range(H):
        x = np.zeros((B, L), dtype=np.complex128)
        x[:, :N] = u[:, h]
        _, uh = _forward_chain(x.reshape([B] + r), Af[h], tw, r)
        _, out = _inverse_chain(uh * shat[h][freq], Ai[h], tw, r)
        y[:, h] = np.real(out.reshape(B, L))[:, :N] / L
    return y


def lbfly_bwd(dy, u, shat, Af, Ai):
    """du [B,H,N] real, dShat [H,L] complex, dAf, dAi [H,S,16,16] complex."""
    dy = np.asarray(dy, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    B, H, N = u.shape
    L = 2 * N
    r, _ = stages(L)
    S = len(r)
    tw, freq = twiddles(L)
    du = np.empty_like(u)
    dshat = np.zeros((H, L), dtype=np.complex128)
    dAf = np.zeros((H, S, 16, 16), dtype=np.complex128)
    dAi = np.zeros((H, S, 16, 16), dtype=np.complex128)
    for h in range(H):
        x = np.zeros((B, L), dtype=np.complex128)
        x[:, :N] = u[:, h]
        xs, uh = _forward_chain(x.reshape([B] + r), Af[h], tw, r)
        sh = shat[h][freq]
        ins, _ = _inverse_chain(uh * sh, Ai[h], tw, r)
        g = np.zeros((B, L), dtype=np.complex128)
        g[:, :N] = dy[:, h] / L
        g = g.reshape([B] + r)
        for s in range(S):                                   # back through the inverse chain, last applied first
            rs = r[s]
            dAi[h, s, :rs, :rs] = _outer(g, ins[s], 1 + s)
            g = _apply(np.conj(Ai[h, s, :rs, :rs]).T, g, 1 + s)
            if s < S - 1:
                g = g * tw[s]
        np.add.at(dshat[h], freq.reshape(-1), np.sum(g * np.conj(uh), axis=0).reshape(-1))
        g = g * np.conj(sh)
        for s in range(S - 1, -1, -1):                       # back through the forward chain
            rs = r[s]
            if s < S - 1:
                g = g * np.conj(tw[s])
            dAf[h, s, :rs, :rs] = _outer(g, xs[s], 1 + s)
            g = _apply(np.conj(Af[h, s, :rs, :rs]).T, g, 1 + s)
        du[:, h] = np.real(g.reshape(B, L))[:, :N]
    return du, dshat, dAf, dAi
