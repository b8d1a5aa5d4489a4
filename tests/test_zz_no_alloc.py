"""The entry point that allocates nothing (longconv_fwd_noalloc), through the C ABI: its output against
longconv_fwd's on two calls in a row, the second with a smaller input (the static scratch array keeps the first
call's contents), for a single-pass and a multi-pass plan, with the spectrum computed on the fly and cached;
a shape beyond the array's size is refused before anything runs."""
from __future__ import annotations

import dataclasses

import numpy as np
import pytest

import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _w(key, **kw):
    return dataclasses.replace(wl.WORKLOADS[key], **kw)


def _both(inp, cached):
    import paper_2302_06646_amd as lc
    from gpu_harness import GpuRun, to_f64
    g = GpuRun(inp)
    ks = g.kspec() if cached else None
    want = g.fwd(kspec=ks).copy()
    y2 = torch.full_like(g.u, float("nan"))
    lc.longconv_fwd_noalloc(g.u, g.k, g.D, y2, kspec=ks)
    torch.cuda.synchronize()
    got = to_f64(y2, g.io)
    assert np.all(np.isfinite(got))
    assert np.array_equal(got, want), "longconv_fwd_noalloc differs from longconv_fwd"
    return g


@pytest.mark.parametrize("cached", [False, True])
def test_no_alloc_forward_matches_longconv_fwd_twice_in_a_row(cached):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    from gpu_harness import TOL
    # first call: B=6, H=40, N=2048 bf16 (wave kernel); second, smaller: B=3, H=5, N=512
    big = wl.generate(_w("2", N=2048), B=6, H=40)
    small = wl.generate(_w("2", N=512), B=3, H=5)
    _both(big, cached)
    g = _both(small, cached)
    ref = oracle.longconv_fwd(small.u, small.k.astype(np.float64), small.D.astype(np.float64))
    assert wl.rel_l2(g.fwd(), ref) <= TOL[small.w.dtype]
    # multi-pass plan (its workspace lives in the array too), then a smaller single-pass fp32 call
    _both(wl.generate(wl.WORKLOADS["4a"], B=2, H=3), cached)
    _both(wl.generate(wl.WORKLOADS["1"], B=1, H=2), cached)


def test_no_alloc_forward_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2302_06646_amd as lc
    B, H, N = 2, 1024, 16384                       # on-the-fly spectrum alone is 128 MiB
    assert lc.longconv_workspace_bytes(B, H, N, lc.F16, False) > lc.STATIC_SCRATCH_BYTES
    u = torch.zeros(B, H, N, dtype=torch.float16, device="cuda")
    y = torch.full_like(u, 5.0)
    k = torch.zeros(H, N, device="cuda")
    D = torch.zeros(H, device="cuda")
    with pytest.raises(lc.LongconvError, match="workspace"):
        lc.longconv_fwd_noalloc(u, k, D, y)
    torch.cuda.synchronize()
    assert bool((y == 5.0).all())                  # nothing was launched
