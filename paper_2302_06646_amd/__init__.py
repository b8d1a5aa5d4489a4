"""Thin Python binding of liblongconv (argument marshalling only).

Every step of the path — spectrum precompute, FFT stages, pointwise product,
inverse, truncation, skip term, gradients — runs inside the HIP kernels of
``liblongconv.so``; PyTorch is used here only to own device memory and to name
the stream.  There is no CPU fallback: if the library is missing, importing
the functions raises.

Functions mirror the C ABI of ``include/longconv.h``:
    longconv_init, longconv_kspec_bytes, longconv_workspace_bytes,
    longconv_kspec_compute, longconv_fwd, longconv_bwd, longconv_plan_string,
    longconv_set_option, longconv_fwd_noalloc, longconv_kreg_fwd, longconv_kreg_bwd,
    longconv_fwd_gated, longconv_bwd_gated, longconv2d_workspace_bytes, longconv2d_fwd, longconv2d_bwd,
    longconv_lbfly_workspace_bytes, longconv_lbfly_spectrum, longconv_lbfly_spectrum_bwd, longconv_lbfly_fwd,
    longconv_lbfly_bwd, longconv_blocksize_fwd
"""
from __future__ import annotations

import ctypes
import os

import torch

F32, F16, BF16 = 0, 1, 2
_TORCH_DTYPE = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}
_CODE = {v: k for k, v in _TORCH_DTYPE.items()}

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblongconv.so")
_lib = None

EXPORTS = ("longconv_init", "longconv_kspec_bytes", "longconv_workspace_bytes",
           "longconv_kspec_compute", "longconv_fwd", "longconv_bwd", "longconv_status_string",
           "longconv_last_hip_error", "longconv_plan_string", "longconv_set_option",
           "longconv_fwd_noalloc", "longconv_kreg_fwd", "longconv_kreg_bwd",
           "longconv_fwd_gated", "longconv_bwd_gated",
           "longconv2d_workspace_bytes", "longconv2d_fwd", "longconv2d_bwd",
           "longconv_lbfly_workspace_bytes", "longconv_lbfly_spectrum", "longconv_lbfly_spectrum_bwd",
           "longconv_lbfly_fwd", "longconv_lbfly_bwd", "longconv_blocksize_fwd")


class LongconvError(RuntimeError):
    pass


def lib():
    """Load liblongconv.so (built by ``python -m paper_2302_06646_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LongconvError(f"{LIB_PATH} not found: build it with "
                                "`python -m paper_2302_06646_amd.build` (no fallback path exists)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int
        L.longconv_init.restype = ci
        L.longconv_kspec_bytes.restype = sz
        L.longconv_kspec_bytes.argtypes = [i64, i64, ci]
        L.longconv_workspace_bytes.restype = sz
        L.longconv_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
        L.longconv_kspec_compute.restype = ci
        L.longconv_kspec_compute.argtypes = [vp, vp, vp, i64, i64, ci, vp, sz, vp]
        L.longconv_fwd.restype = ci
        L.longconv_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, sz, vp]
        L.longconv_fwd_noalloc.restype = ci
        L.longconv_fwd_noalloc.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp]
        L.longconv_bwd.restype = ci
        L.longconv_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, sz, vp]
        L.longconv_status_string.restype = ctypes.c_char_p
        L.longconv_status_string.argtypes = [ci]
        L.longconv_last_hip_error.restype = ctypes.c_char_p
        L.longconv_plan_string.restype = ctypes.c_char_p
        L.longconv_plan_string.argtypes = [i64, ci]
        L.longconv_kreg_fwd.restype = ci
        L.longconv_kreg_fwd.argtypes = [vp, vp, vp, i64, i64, ci, ctypes.c_float, vp]
        L.longconv_kreg_bwd.restype = ci
        L.longconv_kreg_bwd.argtypes = [vp, vp, vp, vp, i64, i64, ci, ctypes.c_float, vp]
        L.longconv_fwd_gated.restype = ci
        L.longconv_fwd_gated.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, sz, vp]
        L.longconv_bwd_gated.restype = ci
        L.longconv_bwd_gated.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, sz, vp]
        L.longconv2d_workspace_bytes.restype = sz
        L.longconv2d_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci]
        L.longconv2d_fwd.restype = ci
        L.longconv2d_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, sz, vp]
        L.longconv2d_bwd.restype = ci
        L.longconv2d_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, sz, vp]
        L.longconv_lbfly_workspace_bytes.restype = sz
        L.longconv_lbfly_workspace_bytes.argtypes = [i64, i64, i64, ci]
        L.longconv_lbfly_spectrum.restype = ci
        L.longconv_lbfly_spectrum.argtypes = [vp, vp, vp, i64, i64, vp]
        L.longconv_lbfly_spectrum_bwd.restype = ci
        L.longconv_lbfly_spectrum_bwd.argtypes = [vp, vp, vp, i64, i64, vp]
        L.longconv_lbfly_fwd.restype = ci
        L.longconv_lbfly_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, vp]
        L.longconv_lbfly_bwd.restype = ci
        L.longconv_lbfly_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, sz, vp]
        L.longconv_blocksize_fwd.restype = ci
        L.longconv_blocksize_fwd.argtypes = [vp, vp, vp, i64, i64, i64, ci, ci, vp]
        L.longconv_set_option.restype = ci
        L.longconv_set_option.argtypes = [ctypes.c_char_p, ci]
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != 0:
        L = lib()
        msg = L.longconv_status_string(status).decode()
        hip = L.longconv_last_hip_error().decode()
        raise LongconvError(f"{what}: {msg}" + (f" [{hip}]" if status == 6 and hip else ""))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _need(t, name, dtype, shape):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise LongconvError(f"{name} must be a contiguous device tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise LongconvError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def dtype_code(t: torch.Tensor) -> int:
    return _CODE[t.dtype]


def longconv_init() -> None:
    _check(lib().longconv_init(), "longconv_init")


def longconv_kspec_bytes(H: int, N: int, io: int) -> int:
    return int(lib().longconv_kspec_bytes(H, N, io))


def longconv_workspace_bytes(B: int, H: int, N: int, io: int, backward) -> int:
    """backward: False / 0 forward, True / 1 backward, 2 gated backward."""
    return int(lib().longconv_workspace_bytes(B, H, N, io, int(backward)))


def longconv_plan_string(N: int, io: int) -> str:
    return lib().longconv_plan_string(N, io).decode()


OPTION_DEFAULTS = {"engine": 0, "inner_log2": 0, "staged_kernel": 0, "fuse_pass_a": 1, "fuse_bwd": 1}


def longconv_set_option(name: str, value: int) -> None:
    """Debug/test switch of the library (see include/longconv.h)."""
    _check(lib().longconv_set_option(name.encode(), int(value)), f"longconv_set_option({name})")


def longconv_kreg_fwd(k, drop_mask, kbar, p: int, lam: float, stream=None) -> None:
    """kbar <- Squash(Smooth(dropout(k))) (Algorithm 1 lines 1-3); drop_mask may be None."""
    H, N = k.shape
    _need(k, "k", torch.float32, (H, N)); _need(drop_mask, "drop_mask", torch.float32, (H, N))
    _need(kbar, "kbar", torch.float32, (H, N))
    _check(lib().longconv_kreg_fwd(_ptr(k), _ptr(drop_mask), _ptr(kbar), H, N, int(p), float(lam), _stream(stream)),
           "longconv_kreg_fwd")


def longconv_kreg_bwd(k, drop_mask, dkbar, dk, p: int, lam: float, stream=None) -> None:
    """dk <- chain rule through dropout, Smooth and Squash applied to dkbar."""
    H, N = k.shape
    _need(k, "k", torch.float32, (H, N)); _need(drop_mask, "drop_mask", torch.float32, (H, N))
    _need(dkbar, "dkbar", torch.float32, (H, N)); _need(dk, "dk", torch.float32, (H, N))
    _check(lib().longconv_kreg_bwd(_ptr(k), _ptr(drop_mask), _ptr(dkbar), _ptr(dk), H, N, int(p), float(lam),
                                   _stream(stream)), "longconv_kreg_bwd")


def new_workspace(B, H, N, io, backward, device="cuda"):
    """Allocate a workspace tensor of the size the library asks for (caller-owned)."""
    n = longconv_workspace_bytes(B, H, N, io, backward)
    if n == 0:
        raise LongconvError("bad shape or dtype")
    return torch.empty(n, dtype=torch.uint8, device=device)


def new_kspec(H, N, io, device="cuda"):
    n = longconv_kspec_bytes(H, N, io)
    if n == 0:
        raise LongconvError("bad shape or dtype")
    return torch.empty(n, dtype=torch.uint8, device=device)


def longconv_kspec_compute(k, D, kspec, io: int, workspace, stream=None) -> None:
    H, N = k.shape
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _check(lib().longconv_kspec_compute(_ptr(k), _ptr(D), _ptr(kspec), H, N, io, _ptr(workspace),
                                        0 if workspace is None else workspace.numel(), _stream(stream)),
           "longconv_kspec_compute")


def longconv_fwd(u, k, D, y, workspace, kspec=None, stream=None) -> None:
    """y <- (u * k)[:N] + D u.  All tensors caller-allocated on the device."""
    B, H, N = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N))
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _check(lib().longconv_fwd(_ptr(u), _ptr(k), _ptr(D), _ptr(kspec), _ptr(y), B, H, N, io,
                              _ptr(workspace), workspace.numel(), _stream(stream)), "longconv_fwd")


def longconv_fwd_gated(u, k, D, g, y, workspace, kspec=None, stream=None) -> None:
    """y <- g * ((u * k)[:N] + D u)."""
    B, H, N = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N))
    _need(g, "g", _TORCH_DTYPE[io], (B, H, N))
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _check(lib().longconv_fwd_gated(_ptr(u), _ptr(k), _ptr(D), _ptr(kspec), _ptr(g), _ptr(y), B, H, N, io,
                                    _ptr(workspace), workspace.numel(), _stream(stream)), "longconv_fwd_gated")


def longconv_bwd_gated(dy, g, u, k, D, du, dk, dD, dg, workspace, kspec=None, stream=None) -> None:
    """du, dk, dD, dg <- gradients of the gated layer (any may be None).  The workspace must hold
    longconv_workspace_bytes(B, H, N, io, 2) bytes."""
    B, H, N = dy.shape
    io = dtype_code(dy)
    for t, name in ((dy, "dy"), (g, "g"), (u, "u"), (du, "du"), (dg, "dg")):
        _need(t, name, _TORCH_DTYPE[io], (B, H, N))
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _need(dk, "dk", torch.float32, (H, N)); _need(dD, "dD", torch.float32, (H,))
    _check(lib().longconv_bwd_gated(_ptr(dy), _ptr(g), _ptr(u), _ptr(k), _ptr(D), _ptr(kspec), _ptr(du), _ptr(dk),
                                    _ptr(dD), _ptr(dg), B, H, N, io, _ptr(workspace), workspace.numel(),
                                    _stream(stream)), "longconv_bwd_gated")


def longconv2d_workspace_bytes(B: int, H: int, N1: int, N2: int, io: int, backward) -> int:
    return int(lib().longconv2d_workspace_bytes(B, H, N1, N2, io, int(bool(backward))))


def new_workspace2d(B, H, N1, N2, io, backward, device="cuda"):
    n = longconv2d_workspace_bytes(B, H, N1, N2, io, backward)
    if n == 0:
        raise LongconvError("bad shape or dtype")
    return torch.empty(n, dtype=torch.uint8, device=device)


def longconv2d_fwd(u, k, D, y, workspace, stream=None) -> None:
    """y[b,h] <- the 2-D linear convolution of u[b,h] with k[h], truncated to the image, + D[h] u[b,h]."""
    B, H, N1, N2 = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N1, N2)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N1, N2))
    _need(k, "k", torch.float32, (H, N1, N2)); _need(D, "D", torch.float32, (H,))
    _check(lib().longconv2d_fwd(_ptr(u), _ptr(k), _ptr(D), _ptr(y), B, H, N1, N2, io, _ptr(workspace),
                                workspace.numel(), _stream(stream)), "longconv2d_fwd")


def longconv2d_bwd(dy, u, k, D, du, dk, dD, workspace, stream=None) -> None:
    """du, dk, dD <- adjoints of longconv2d_fwd (any of the three may be None)."""
    B, H, N1, N2 = dy.shape
    io = dtype_code(dy)
    for t, name in ((dy, "dy"), (u, "u"), (du, "du")):
        _need(t, name, _TORCH_DTYPE[io], (B, H, N1, N2))
    _need(k, "k", torch.float32, (H, N1, N2)); _need(D, "D", torch.float32, (H,))
    _need(dk, "dk", torch.float32, (H, N1, N2)); _need(dD, "dD", torch.float32, (H,))
    _check(lib().longconv2d_bwd(_ptr(dy), _ptr(u), _ptr(k), _ptr(D), _ptr(du), _ptr(dk), _ptr(dD), B, H, N1, N2, io,
                                _ptr(workspace), workspace.numel(), _stream(stream)), "longconv2d_bwd")


def longconv_lbfly_workspace_bytes(B: int, H: int, N: int, io: int) -> int:
    return int(lib().longconv_lbfly_workspace_bytes(B, H, N, io))


def longconv_lbfly_spectrum(k, D, shat, stream=None) -> None:
    """shat [H, 2N, 2] <- FFT([k, 0]) + D in natural frequency order (re, im)."""
    H, N = k.shape
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _need(shat, "shat", torch.float32, (H, 2 * N, 2))
    _check(lib().longconv_lbfly_spectrum(_ptr(k), _ptr(D), _ptr(shat), H, N, _stream(stream)), "longconv_lbfly_spectrum")


def longconv_lbfly_spectrum_bwd(dshat, dk, dD, stream=None) -> None:
    """dk [H, N], dD [H] <- the adjoint of longconv_lbfly_spectrum applied to dshat (either may be None)."""
    H, L, _ = dshat.shape
    _need(dshat, "dshat", torch.float32, (H, L, 2)); _need(dk, "dk", torch.float32, (H, L // 2))
    _need(dD, "dD", torch.float32, (H,))
    _check(lib().longconv_lbfly_spectrum_bwd(_ptr(dshat), _ptr(dk), _ptr(dD), H, L // 2, _stream(stream)),
           "longconv_lbfly_spectrum_bwd")


def longconv_lbfly_fwd(u, shat, Af, Ai, y, stream=None) -> None:
    """y <- Re(T_B(shat . T_A([u, 0])))[:N] with the per-head blocks Af, Ai [H, 3, 16, 16, 2]."""
    B, H, N = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N))
    _need(shat, "shat", torch.float32, (H, 2 * N, 2))
    _need(Af, "Af", torch.float32, (H, 3, 16, 16, 2)); _need(Ai, "Ai", torch.float32, (H, 3, 16, 16, 2))
    _check(lib().longconv_lbfly_fwd(_ptr(u), _ptr(shat), _ptr(Af), _ptr(Ai), _ptr(y), B, H, N, io, _stream(stream)),
           "longconv_lbfly_fwd")


def longconv_lbfly_bwd(dy, u, shat, Af, Ai, du, dshat, dAf, dAi, workspace, stream=None) -> None:
    """du, dshat, dAf, dAi <- gradients of longconv_lbfly_fwd (any may be None)."""
    B, H, N = dy.shape
    io = dtype_code(dy)
    for t, name in ((dy, "dy"), (u, "u"), (du, "du")):
        _need(t, name, _TORCH_DTYPE[io], (B, H, N))
    _need(shat, "shat", torch.float32, (H, 2 * N, 2)); _need(dshat, "dshat", torch.float32, (H, 2 * N, 2))
    for t, name in ((Af, "Af"), (Ai, "Ai"), (dAf, "dAf"), (dAi, "dAi")):
        _need(t, name, torch.float32, (H, 3, 16, 16, 2))
    _check(lib().longconv_lbfly_bwd(_ptr(dy), _ptr(u), _ptr(shat), _ptr(Af), _ptr(Ai), _ptr(du), _ptr(dshat),
                                    _ptr(dAf), _ptr(dAi), B, H, N, io, _ptr(workspace), workspace.numel(),
                                    _stream(stream)), "longconv_lbfly_bwd")


def longconv_blocksize_fwd(u, shat, y, log2r: int, stream=None) -> None:
    """y <- the convolution computed with DFT blocks of 2**log2r points per stage (block-size study)."""
    B, H, N = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N))
    _need(shat, "shat", torch.float32, (H, 2 * N, 2))
    _check(lib().longconv_blocksize_fwd(_ptr(u), _ptr(shat), _ptr(y), B, H, N, io, int(log2r), _stream(stream)),
           "longconv_blocksize_fwd")


STATIC_SCRATCH_BYTES = 64 << 20


def longconv_fwd_noalloc(u, k, D, y, kspec=None, stream=None) -> None:
    """longconv_fwd without a workspace argument: scratch is the library's static device array."""
    B, H, N = u.shape
    io = dtype_code(u)
    _need(u, "u", _TORCH_DTYPE[io], (B, H, N)); _need(y, "y", _TORCH_DTYPE[io], (B, H, N))
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _check(lib().longconv_fwd_noalloc(_ptr(u), _ptr(k), _ptr(D), _ptr(kspec), _ptr(y), B, H, N, io,
                                      _stream(stream)), "longconv_fwd_noalloc")


def longconv_bwd(dy, u, k, D, du, dk, dD, workspace, kspec=None, stream=None) -> None:
    """du, dk, dD <- adjoints (any of the three may be None to skip it)."""
    B, H, N = dy.shape
    io = dtype_code(dy)
    _need(dy, "dy", _TORCH_DTYPE[io], (B, H, N)); _need(u, "u", _TORCH_DTYPE[io], (B, H, N))
    _need(du, "du", _TORCH_DTYPE[io], (B, H, N))
    _need(k, "k", torch.float32, (H, N)); _need(D, "D", torch.float32, (H,))
    _need(dk, "dk", torch.float32, (H, N)); _need(dD, "dD", torch.float32, (H,))
    _check(lib().longconv_bwd(_ptr(dy), _ptr(u), _ptr(k), _ptr(D), _ptr(kspec), _ptr(du), _ptr(dk), _ptr(dD),
                              B, H, N, io, _ptr(workspace), workspace.numel(), _stream(stream)), "longconv_bwd")
