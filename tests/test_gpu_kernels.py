"""Kernel-level parity on the GPU: the tile contraction (every operand layout, tile shape
and dtype, ragged sizes), the implicit-GEMM convolution passes and the kernels of the ViT-shaped
stages (LayerNorm, GELU, attention core) against the oracle."""
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


LARGE_TILE_CASES = [
    # pass, B, H, W, Cin, Cout, ks, stride, pad: shapes that fill the chip with 256 x 256 tiles
    ("fwd", 16, 56, 56, 64, 256, 3, 1, 1),
    ("dgrad", 16, 56, 56, 256, 64, 3, 1, 1),
    ("fwd", 64, 56, 56, 64, 256, 3, 2, 1),       # stride 2: padding on one side only
    ("dgrad", 16, 56, 56, 256, 64, 3, 2, 1),     # stride 2: taps on the stride lattice
    ("dgrad", 4, 45, 45, 4040, 128, 1, 1, 0),    # ragged in both directions
    ("fwd", 8, 28, 28, 1024, 2048, 1, 1, 0),     # 16 slabs
    ("fwd", 2, 9, 7, 64, 64, 3, 1, 1),           # a single ragged tile
    ("dgrad", 3, 10, 10, 64, 128, 3, 2, 1),
]


@pytest.mark.parametrize("tile", [256, 128])
@pytest.mark.parametrize("case", LARGE_TILE_CASES)
def test_conv_large_tile_matches_oracle(case, tile):
    """Forward / data gradient on the direct-to-LDS kernel (bf16; swizzled rows, two stages), 256 x 256 and
    128 x 128 tiles, against the oracle's convolution."""
    torch = _torch()
    which, B, H, W, Cin, Cout, ks, st, pad = case
    dtype = wl.BF16
    x = wl.random_normal(7, 1, B * H * W * Cin).reshape(B, H, W, Cin)
    w = wl.random_normal(7, 2, Cout * ks * ks * Cin).reshape(Cout, ks, ks, Cin) / np.sqrt(ks * ks * Cin)
    xr, wr = _rnd(x, dtype), _rnd(w, dtype)
    if which == "fwd":
        ref = L.conv2d_fwd(xr, wr, st, pad)
        xd, wd = _dev(x, dtype), _dev(w, dtype)
        got = torch.full(ref.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        b.cdp_k_conv(dtype, 3 if tile == 256 else 5, xd.data_ptr(), wd.data_ptr(), got.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    else:
        Ho, Wo = (H + 2 * pad - ks) // st + 1, (W + 2 * pad - ks) // st + 1
        dy = wl.random_normal(7, 3, B * Ho * Wo * Cout).reshape(B, Ho, Wo, Cout)
        ref, _ = L.conv2d_bwd(xr, wr, st, pad, _rnd(dy, dtype))
        dyd, wtd = _dev(dy, dtype), _dev(np.transpose(w, (3, 1, 2, 0)), dtype)
        got = torch.full(x.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
        b.cdp_k_conv(dtype, 4 if tile == 256 else 6, dyd.data_ptr(), wtd.data_ptr(), got.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    torch.cuda.synchronize()
    g = got.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(g).all()
    assert np.abs(g - ref).max() / np.abs(ref).max() <= 2.0 ** -7


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


def _close(got, ref, tol, what):
    g = got.float().cpu().numpy().astype(np.float64).reshape(ref.shape)
    assert np.isfinite(g).all(), what
    err = np.abs(g - ref).max() / max(1e-6, np.abs(ref).max())
    assert err <= tol, (what, err)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("rows,C", [(6272, 768), (100, 20), (37, 1000), (5, 3)])
def test_layernorm_kernels_match_oracle(dtype, rows, C):
    """Forward and backward (with a residual addend and running gamma / beta sums) at the
    ViT-B/16 shape and at ragged ones (rows that are not whole 16-byte chunks take the
    element-wise kernels)."""
    torch = _torch()
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    x = wl.random_normal(7, 1, rows * C).reshape(rows, C) * 1.5 + 0.3
    dy = wl.random_normal(7, 2, rows * C).reshape(rows, C)
    add = wl.random_normal(7, 3, rows * C).reshape(rows, C)
    gamma = 1.0 + 0.2 * wl.random_normal(7, 4, C)
    beta = 0.1 * wl.random_normal(7, 5, C)
    g0, b0 = wl.random_normal(7, 6, C), wl.random_normal(7, 7, C)   # running sums the backward adds to
    xr, dyr, addr = _rnd(x, dtype), _rnd(dy, dtype), _rnd(add, dtype)
    gam, bet = _rnd(gamma, wl.F32), _rnd(beta, wl.F32)
    y = L.layernorm_fwd(xr, gam, bet)
    dx, dg, db = L.layernorm_bwd(xr, gam, dyr)
    xd, dyd, addd = _dev(x, dtype), _dev(dy, dtype), _dev(add, dtype)
    gd, bd = _dev(gamma, wl.F32), _dev(beta, wl.F32)
    yd = torch.full((rows, C), float("nan"), dtype=tdt, device="cuda")
    b.cdp_k_layernorm(dtype, 0, xd.data_ptr(), 0, 0, gd.data_ptr(), bd.data_ptr(), yd.data_ptr(), 0, 0, 0, 0, rows, C)
    dxd = torch.full((rows, C), float("nan"), dtype=tdt, device="cuda")
    dgd, dbd = _dev(g0, wl.F32), _dev(b0, wl.F32)
    ws = torch.full((2 * rows + 2 * C * ((rows + 31) // 32) + 64,), float("nan"), dtype=torch.float32, device="cuda")
    b.cdp_k_layernorm(dtype, 1, xd.data_ptr(), dyd.data_ptr(), addd.data_ptr(), gd.data_ptr(), 0, dxd.data_ptr(),
                      dgd.data_ptr(), dbd.data_ptr(), ws.data_ptr(), ws.numel() * 4, rows, C)
    torch.cuda.synchronize()
    tol = 2.0 ** -7 if dtype == wl.BF16 else 1e-5
    _close(yd, y, tol, "y")
    _close(dxd, dx + addr, tol, "dx")
    _close(dgd, _rnd(g0, wl.F32) + dg, 1e-5, "dgamma")
    _close(dbd, _rnd(b0, wl.F32) + db, 1e-5, "dbeta")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_gelu_kernels_match_oracle(dtype):
    torch = _torch()
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    n = 1000003   # not a multiple of the vector width: the tail runs element by element
    x = wl.random_normal(8, 1, n) * 2.0
    dy = wl.random_normal(8, 2, n)
    xr, dyr = _rnd(x, dtype), _rnd(dy, dtype)
    xd, dyd = _dev(x, dtype), _dev(dy, dtype)
    yd = torch.full((n,), float("nan"), dtype=tdt, device="cuda")
    dxd = torch.full((n,), float("nan"), dtype=tdt, device="cuda")
    b.cdp_k_gelu(dtype, 0, xd.data_ptr(), 0, yd.data_ptr(), n)
    b.cdp_k_gelu(dtype, 1, xd.data_ptr(), dyd.data_ptr(), dxd.data_ptr(), n)
    torch.cuda.synchronize()
    tol = 2.0 ** -7 if dtype == wl.BF16 else 2e-6
    _close(yd, L.gelu_fwd(xr), tol, "gelu")
    _close(dxd, L.gelu_bwd(xr, dyr), tol, "dgelu")


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
@pytest.mark.parametrize("B,T,D,heads", [(2, 196, 768, 12), (3, 9, 20, 4), (1, 324, 16, 2), (2, 16, 32, 4), (2, 50, 64, 2),
                                         (1, 256, 128, 2), (1, 33, 64, 1), (1, 70, 160, 2), (2, 129, 48, 3), (1, 200, 96, 1),
                                         (1, 260, 64, 2)])
def test_attention_kernels_match_oracle(dtype, B, T, D, heads):
    """Probabilities, output and the gradient with respect to q | k | v: the ViT-B/16 shape,
    a shape where nothing is a multiple of four (element-wise staging, ragged tiles), 324
    tokens, the reduced test shape, heads of width 32 / 64 with 50, 256 and 33 tokens, and the limits of the
    one-kernel score rows of the bf16 path (head widths 80, 16 and 96: the last one too wide for it; 129 and 260
    tokens: a third key block of one key, and one token too many)."""
    torch = _torch()
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    eb = 2 if dtype == wl.BF16 else 4
    qkv = wl.random_normal(9, 1, B * T * 3 * D).reshape(B, 1, T, 3 * D)
    dout = wl.random_normal(9, 2, B * T * D).reshape(B, 1, T, D)
    qr, dor = _rnd(qkv, dtype), _rnd(dout, dtype)
    # the stored probabilities and the stored score gradient carry the element type's rounding
    P = _rnd(L.attention_probs(qr, heads), dtype)
    out = L.attention_apply(qr, P, heads)
    dqkv = L.attention_input_grad(qr, P, _rnd(L.attention_score_grad(qr, P, heads, dor), dtype), heads, dor)
    qd, dod = _dev(qkv, dtype), _dev(dout, dtype)
    tt = B * heads * T * T
    Pd = torch.full((B, heads, T, T), float("nan"), dtype=tdt, device="cuda")
    outd = torch.full((B, T, D), float("nan"), dtype=tdt, device="cuda")
    dqd = torch.full((B, T, 3 * D), float("nan"), dtype=tdt, device="cuda")
    ws = torch.full((2 * tt + 128,), float("nan"), dtype=torch.float32, device="cuda")
    b.cdp_k_attention(dtype, 0, qd.data_ptr(), Pd.data_ptr(), 0, outd.data_ptr(), ws.data_ptr(), ws.numel() * 4, B, T, D, heads)
    b.cdp_k_attention(dtype, 1, qd.data_ptr(), Pd.data_ptr(), dod.data_ptr(), dqd.data_ptr(), ws.data_ptr(), ws.numel() * 4,
                      B, T, D, heads)
    torch.cuda.synchronize()
    tol = 2.0 ** -6 if dtype == wl.BF16 else 2e-5
    _close(Pd, P, tol, "P")
    _close(outd, out, tol, "out")
    _close(dqd, dqkv, tol, "dqkv")

