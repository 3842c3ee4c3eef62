"""Kernel-level parity on the GPU: the tile contraction (every operand layout, tile shape
and dtype, ragged sizes) and the implicit-GEMM convolution passes against the oracle."""
import numpy as np
import pytest

import cdp_workloads as wl
from oracle import layers as L
from paper_2403_08837_amd import binding as b

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _dev(a, dtype):
    torch = _torch()
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == wl.BF16 else t.contiguous()


def _rnd(a, dtype):
    return L.round_bf16(a) if dtype == wl.BF16 else np.asarray(a, dtype=np.float32).astype(np.float64)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("shape", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("a_k,b_k", [(1, 1), (0, 0), (1, 0), (0, 1)])
@pytest.mark.parametrize("M,N,K", [(8, 64, 64), (64, 200, 136), (130, 257, 70), (333, 129, 515), (5, 7, 3), (32, 300, 1100),
                                   (32, 1024, 1024), (17, 200, 3072), (32, 96, 136), (1, 40, 8), (9, 33, 2056)])
def test_gemm_all_layouts(dtype, shape, a_k, b_k, M, N, K):
    torch = _torch()
    if shape >= 3 and not (a_k and b_k):
        pytest.skip("the weight-streaming kernel takes k-contiguous operands only")
    A = wl.random_normal(1, 10 * M + K, M * K).reshape(M, K)
    Bm = wl.random_normal(2, 10 * N + K, N * K).reshape(N, K)
    ref = _rnd(A, dtype) @ _rnd(Bm, dtype).T
    Ad = _dev(A if a_k else A.T, dtype)
    Bd = _dev(Bm if b_k else Bm.T, dtype)
    Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    b.cdp_k_gemm(dtype, shape, a_k, b_k, Ad.data_ptr(), Bd.data_ptr(), Cd.data_ptr(), M, N, K,
                 K if a_k else M, K if b_k else N)
    torch.cuda.synchronize()
    got = Cd.cpu().numpy().astype(np.float64)
    tol = 2e-5 * np.sqrt(K) * max(1.0, np.abs(ref).max())
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= tol, np.abs(got - ref).max()


CONV_CASES = [
    # B, H, W, Cin, Cout, ks, stride, pad
    (2, 8, 8, 8, 16, 3, 1, 1),
    (3, 9, 7, 16, 8, 3, 2, 1),
    (2, 12, 12, 3, 8, 7, 2, 3),     # stem-like: Cin = 3 takes the element-wise gather path
    (2, 8, 8, 3, 8, 3, 1, 1),
    (4, 6, 6, 32, 64, 1, 1, 0),
    (4, 6, 6, 32, 64, 1, 2, 0),
    (2, 16, 16, 64, 64, 3, 1, 1),
    (1, 5, 5, 24, 40, 3, 1, 1),     # channel counts that are multiples of 8 but not of the tile
]


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_passes_match_oracle(dtype, case):
    torch = _torch()
    B, H, W, Cin, Cout, ks, st, pad = case
    x = wl.random_normal(3, 1, B * H * W * Cin).reshape(B, H, W, Cin)
    w = wl.random_normal(3, 2, Cout * ks * ks * Cin).reshape(Cout, ks, ks, Cin) / np.sqrt(ks * ks * Cin)
    xr, wr = _rnd(x, dtype), _rnd(w, dtype)
    y = L.conv2d_fwd(xr, wr, st, pad)
    dy = wl.random_normal(3, 3, y.size).reshape(y.shape)
    dyr = _rnd(dy, dtype)
    dx, dw = L.conv2d_bwd(xr, wr, st, pad, dyr)
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    tol_out = 2.0 ** -7 if dtype == wl.BF16 else 1e-5

    xd, wd, dyd = _dev(x, dtype), _dev(w, dtype), _dev(dy, dtype)
    yd = torch.full(y.shape, float("nan"), dtype=tdt, device="cuda")
    b.cdp_k_conv(dtype, 0, xd.data_ptr(), wd.data_ptr(), yd.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    wtd = _dev(np.transpose(w, (3, 1, 2, 0)), dtype)        # [Cin][k][k][Cout]
    dxd = torch.full(x.shape, float("nan"), dtype=tdt, device="cuda")
    b.cdp_k_conv(dtype, 1, dyd.data_ptr(), wtd.data_ptr(), dxd.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    dwd = torch.full(w.shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.full((w.size * (y.size // Cout // 1024 + 4),), float("nan"), dtype=torch.float32, device="cuda")
    b.cdp_k_conv(dtype, 2, dyd.data_ptr(), xd.data_ptr(), dwd.data_ptr(), B, H, W, Cin, Cout, ks, st, pad,
                 ws.data_ptr(), ws.numel() * 4)
    dw2 = torch.full(w.shape, float("nan"), dtype=torch.float32, device="cuda")      # single-pass kernel, no workspace
    b.cdp_k_conv(dtype, 2, dyd.data_ptr(), xd.data_ptr(), dw2.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    torch.cuda.synchronize()
    for name, got, ref, tol in (("fwd", yd, y, tol_out), ("dgrad", dxd, dx, tol_out), ("wgrad", dwd, dw, 1e-5),
                                ("wgrad-1pass", dw2, dw, 1e-5)):
        g = got.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all(), name
        err = np.abs(g - ref).max() / max(1e-6, np.abs(ref).max())
        assert err <= tol, (name, err)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("which", ["fwd", "dgrad"])
def test_conv_gemm_many_tiles(dtype, which):
    """A 1x1 convolution with 8100 positions and 4040 output (forward) or input (data gradient)
    channels: about two thousand of the largest tiles (several rounds over the chip), ragged in
    both directions."""
    torch = _torch()
    B, H, W = 4, 45, 45
    Cin, Cout = (128, 4040) if which == "fwd" else (4040, 128)
    x = wl.random_normal(5, 1, B * H * W * Cin).reshape(B, H, W, Cin)
    w = wl.random_normal(5, 2, Cout * Cin).reshape(Cout, 1, 1, Cin) / np.sqrt(Cin)
    xr, wr = _rnd(x, dtype), _rnd(w, dtype)
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    tol = 2.0 ** -7 if dtype == wl.BF16 else 1e-5
    if which == "fwd":
        ref = L.conv2d_fwd(xr, wr, 1, 0)
        xd, wd = _dev(x, dtype), _dev(w, dtype)
        got = torch.full(ref.shape, float("nan"), dtype=tdt, device="cuda")
        b.cdp_k_conv(dtype, 0, xd.data_ptr(), wd.data_ptr(), got.data_ptr(), B, H, W, Cin, Cout, 1, 1, 0)
    else:
        dy = wl.random_normal(5, 3, B * H * W * Cout).reshape(B, H, W, Cout)
        dyr = _rnd(dy, dtype)
        ref, _ = L.conv2d_bwd(xr, wr, 1, 0, dyr)
        dyd, wtd = _dev(dy, dtype), _dev(np.transpose(w, (3, 1, 2, 0)), dtype)
        got = torch.full(x.shape, float("nan"), dtype=tdt, device="cuda")
        b.cdp_k_conv(dtype, 1, dyd.data_ptr(), wtd.data_ptr(), got.data_ptr(), B, H, W, Cin, Cout, 1, 1, 0)
    torch.cuda.synchronize()
    g = got.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(g).all()
    assert np.abs(g - ref).max() / np.abs(ref).max() <= tol

