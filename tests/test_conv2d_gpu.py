"""2-D long convolution through the C ABI against the float64 oracle of direct sums: image sizes whose padded
row-major length lands in every plan family of the 1-D path, all three I/O dtypes, optional outputs, error codes."""
import numpy as np
import pytest
import torch

import paper_2302_06646_amd as lc
import workloads as wl
from gpu_harness import TOL, _compare, to_dev, to_f64
from oracle import conv2d

pytestmark = pytest.mark.gpu


def _inputs(B, H, N1, N2, io, seed=0):
    """Images and output gradients of unit variance; filters that decay away from the origin along both axes (the
    2-D analogue of the decaying 1-D filters of the other tests), scaled so the output has the input's order."""
    r_u, r_k, r_D, r_dy = np.random.default_rng(77000 + 131 * N1 + N2 + seed).spawn(4)
    u_s, u_v = wl.quantize(r_u.standard_normal((B, H, N1, N2), dtype=np.float32), io)
    dy_s, dy_v = wl.quantize(r_dy.standard_normal((B, H, N1, N2), dtype=np.float32), io)
    p = np.arange(N1, dtype=np.float64)[:, None] / N1
    q = np.arange(N2, dtype=np.float64)[None, :] / N2
    k = (r_k.standard_normal((H, N1, N2)) * np.exp(-4.0 * (p + q)) / np.sqrt(N1 * N2 / 16.0)).astype(np.float32)
    D = r_D.standard_normal(H).astype(np.float32)
    return u_s, u_v, dy_s, dy_v, k, D


def _run(u_s, dy_s, k, D, io, want=(True, True, True)):
    B, H, N1, N2 = u_s.shape
    u, dy = to_dev(u_s, io), to_dev(dy_s, io)
    kd, Dd = torch.from_numpy(k).cuda(), torch.from_numpy(D).cuda()
    y, du = torch.full_like(u, float("nan")), torch.full_like(u, float("nan"))
    dk, dD = torch.full_like(kd, float("nan")), torch.full_like(Dd, float("nan"))
    ws = lc.new_workspace2d(B, H, N1, N2, io, True)
    ws.fill_(0xFF)           # NaN patterns in every dtype: nothing may depend on what the workspace held
    lc.longconv2d_fwd(u, kd, Dd, y, ws)
    lc.longconv2d_bwd(dy, u, kd, Dd, du if want[0] else None, dk if want[1] else None, dD if want[2] else None, ws)
    torch.cuda.synchronize()
    return (to_f64(y, io), to_f64(du, io), dk.cpu().numpy().astype(np.float64), dD.cpu().numpy().astype(np.float64))


# (N1, N2, io, B, H): the padded sequence length 2 N1 N2 is 256, 256, 2048, 2048, 8192, 16384, 32768, 131072
CASES = [(16, 8, wl.F32, 3, 2), (1, 128, wl.BF16, 2, 3), (32, 32, wl.BF16, 5, 3), (32, 32, wl.F32, 2, 2),
         (64, 64, wl.F16, 3, 2), (128, 64, wl.BF16, 2, 2), (8, 2048, wl.F16, 2, 2), (256, 256, wl.BF16, 1, 1)]


@pytest.mark.parametrize("N1,N2,io,B,H", CASES)
def test_conv2d_against_the_oracle(N1, N2, io, B, H):
    print(f"[conv2d] N1={N1} N2={N2} io={wl.DTYPE_NAMES[io]} B={B} H={H}", flush=True)
    u_s, u_v, dy_s, dy_v, k, D = _inputs(B, H, N1, N2, io)
    y, du, dk, dD = _run(u_s, dy_s, k, D, io)
    k64, D64 = k.astype(np.float64), D.astype(np.float64)
    ry = conv2d.conv2d_fwd(u_v, k64, D64)
    rdu, rdk, rdD = conv2d.conv2d_bwd(dy_v, u_v, k64, D64)
    flat = lambda a: a.reshape(a.shape[:-2] + (N1 * N2,))      # one image is one "row" of the per-row check
    _compare({"y": flat(y), "du": flat(du), "dk": flat(dk), "dD": dD},
             {"y": flat(ry), "du": flat(rdu), "dk": flat(rdk), "dD": rdD}, TOL[io],
             f"conv2d {N1}x{N2} io={wl.DTYPE_NAMES[io]}")


def test_full_size_image_batch_on_sampled_heads():
    """B=64, H=256, 32x32 bf16 images (the shape timed in the design notes), all of it through the library; eight heads
    (first, last, seeded ones) in full against the oracle."""
    B, H, N1, N2, io = 64, 256, 32, 32, wl.BF16
    u_s, u_v, dy_s, dy_v, k, D = _inputs(B, H, N1, N2, io, seed=3)
    y, du, dk, dD = _run(u_s, dy_s, k, D, io)
    heads = sorted({0, H - 1, *np.random.default_rng(6).choice(H, size=6, replace=False).tolist()})
    k64, D64 = k[heads].astype(np.float64), D[heads].astype(np.float64)
    ry = conv2d.conv2d_fwd(u_v[:, heads], k64, D64)
    rdu, rdk, rdD = conv2d.conv2d_bwd(dy_v[:, heads], u_v[:, heads], k64, D64)
    flat = lambda a: a.reshape(a.shape[:-2] + (N1 * N2,))
    _compare({"y": flat(y[:, heads]), "du": flat(du[:, heads]), "dk": flat(dk[heads]), "dD": dD[heads]},
             {"y": flat(ry), "du": flat(rdu), "dk": flat(rdk), "dD": rdD}, TOL[io], "conv2d full size")
    assert np.all(np.isfinite(y)) and np.all(np.isfinite(du)) and np.all(np.isfinite(dk))


def test_delta_filter_shifts_the_image_exactly():
    # k = delta at (3, 5), D = 0: y is u moved down 3 and right 5, with zeros (not wrapped samples) coming in
    B, H, N1, N2, io = 2, 2, 32, 32, wl.F32
    u_s, u_v, dy_s, dy_v, k, D = _inputs(B, H, N1, N2, io, seed=1)
    k[:] = 0
    k[:, 3, 5] = 1.0
    D[:] = 0
    y, du, dk, dD = _run(u_s, dy_s, k, D, io)
    ref = np.zeros_like(u_v)
    ref[:, :, 3:, 5:] = u_v[:, :, :-3, :-5]
    assert np.max(np.abs(y - ref)) <= 1e-5
    assert np.max(np.abs(y[:, :, :3, :])) <= 1e-5 and np.max(np.abs(y[:, :, :, :5])) <= 1e-5


def test_optional_outputs_and_error_codes():
    B, H, N1, N2, io = 2, 2, 32, 32, wl.BF16
    u_s, u_v, dy_s, dy_v, k, D = _inputs(B, H, N1, N2, io, seed=2)
    k64, D64 = k.astype(np.float64), D.astype(np.float64)
    rdu, rdk, rdD = conv2d.conv2d_bwd(dy_v, u_v, k64, D64)
    y, du, dk, dD = _run(u_s, dy_s, k, D, io, want=(True, False, False))
    assert np.all(np.isnan(dk)) and np.all(np.isnan(dD)) and wl.rel_l2(du, rdu) <= TOL[io]
    y, du, dk, dD = _run(u_s, dy_s, k, D, io, want=(False, True, False))
    assert np.all(np.isnan(du)) and np.all(np.isnan(dD)) and wl.rel_l2(dk, rdk) <= TOL[io]
    y, du, dk, dD = _run(u_s, dy_s, k, D, io, want=(False, False, True))
    assert np.all(np.isnan(du)) and np.all(np.isnan(dk)) and wl.rel_l2(dD, rdD) <= 1e-5
    # shapes the construction does not cover are refused before anything is launched
    assert lc.longconv2d_workspace_bytes(1, 1, 32, 4, io, False) == 0          # rows shorter than one vector
    assert lc.longconv2d_workspace_bytes(1, 1, 24, 32, io, False) == 0         # not a power of two
    assert lc.longconv2d_workspace_bytes(1, 1, 512, 256, io, False) == 0       # 2 N1 N2 above the 1-D limit
    assert lc.longconv2d_workspace_bytes(1, 1, 2, 32, io, False) == 0          # 2 N1 N2 below the 1-D limit
    u, kd, Dd = to_dev(u_s, io), torch.from_numpy(k).cuda(), torch.from_numpy(D).cuda()
    small = torch.empty(lc.longconv2d_workspace_bytes(B, H, N1, N2, io, False) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(lc.LongconvError, match="workspace"):
        lc.longconv2d_fwd(u, kd, Dd, torch.empty_like(u), small)
    assert lc.longconv2d_workspace_bytes(B, H, N1, N2, io, True) > lc.longconv2d_workspace_bytes(B, H, N1, N2, io, False)
