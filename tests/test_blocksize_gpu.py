"""Block-size study kernel through the C ABI: with every block size the result is the plain convolution of the
float64 oracle, to the bound of the fixed path."""
import numpy as np
import pytest
import torch

import oracle
import paper_2302_06646_amd as lc
import workloads as wl
from gpu_harness import TOL, _compare, to_dev, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N", [1024, 4096])
@pytest.mark.parametrize("log2r", [1, 2, 3, 4, 5, 6, 8])
def test_every_block_size_gives_the_convolution(N, log2r):
    if log2r == 8 and N != 4096:
        pytest.skip("256-point blocks are built for N = 4096 only (the call is refused, see test_refused_arguments)")
    B, H = 5, 3
    print(f"[blocksize] N={N} r={1 << log2r}", flush=True)
    w = wl.Workload(6, B, H, N, wl.F16, "decay_alpha_squash")
    inp = wl.generate(w, seed_extra=log2r)
    u = to_dev(inp.u_store, wl.F16)
    k, D = torch.from_numpy(inp.k).cuda(), torch.from_numpy(inp.D).cuda()
    shat = torch.full((H, 2 * N, 2), float("nan"), device="cuda")
    lc.longconv_lbfly_spectrum(k, D, shat)
    y = torch.full_like(u, float("nan"))
    lc.longconv_blocksize_fwd(u, shat, y, log2r)
    torch.cuda.synchronize()
    ref = oracle.longconv_fwd(inp.u, inp.k.astype(np.float64), inp.D.astype(np.float64))
    _compare({"y": to_f64(y, wl.F16)}, {"y": ref}, TOL[wl.F16], f"block size {1 << log2r} N={N}")


@pytest.mark.parametrize("log2r,N,B,H", [(6, 4096, 1, 1), (6, 1024, 3, 2), (6, 1024, 17, 5), (8, 4096, 1, 1), (8, 4096, 7, 40),
                                         (6, 4096, 9, 33)])
def test_dense_blocks_on_odd_shapes(log2r, N, B, H):
    # the dense-block kernels keep several rows resident: row counts that do not fill a group, single rows, more
    # workgroups than compute units
    print(f"[blocksize] N={N} r={1 << log2r} B={B} H={H}", flush=True)
    w = wl.Workload(6, B, H, N, wl.F16, "decay_alpha_squash")
    inp = wl.generate(w, seed_extra=100 + log2r)
    u = to_dev(inp.u_store, wl.F16)
    k, D = torch.from_numpy(inp.k).cuda(), torch.from_numpy(inp.D).cuda()
    shat = torch.empty((H, 2 * N, 2), device="cuda")
    lc.longconv_lbfly_spectrum(k, D, shat)
    y = torch.full_like(u, float("nan"))
    lc.longconv_blocksize_fwd(u, shat, y, log2r)
    torch.cuda.synchronize()
    ref = oracle.longconv_fwd(inp.u, inp.k.astype(np.float64), inp.D.astype(np.float64))
    _compare({"y": to_f64(y, wl.F16)}, {"y": ref}, TOL[wl.F16], f"block size {1 << log2r} N={N} B={B} H={H}")


def test_refused_arguments():
    u = torch.zeros(2, 2, 1024, device="cuda", dtype=torch.float16)
    shat = torch.zeros(2, 2048, 2, device="cuda")
    with pytest.raises(lc.LongconvError, match="shape"):
        lc.longconv_blocksize_fwd(u, shat, torch.empty_like(u), 7)
    with pytest.raises(lc.LongconvError, match="shape"):
        lc.longconv_blocksize_fwd(u, shat, torch.empty_like(u), 8)       # 256-point blocks: N = 4096 only
    ub = u.to(torch.bfloat16)
    with pytest.raises(lc.LongconvError, match="dtype"):
        lc.longconv_blocksize_fwd(ub, shat, torch.empty_like(ub), 4)
    u2 = torch.zeros(2, 2, 2048, device="cuda", dtype=torch.float16)
    with pytest.raises(lc.LongconvError, match="shape"):
        lc.longconv_blocksize_fwd(u2, torch.zeros(2, 4096, 2, device="cuda"), torch.empty_like(u2), 4)
