#!/usr/bin/env python3
"""Times single contractions through the kernel-level C ABI (cdp_k_gemm / cdp_k_conv) on the
shapes the five workloads are made of, and prints achieved TFLOP/s and GB/s per shape.

  python -m paper_2403_08837_amd.kernel_bench            # bf16, all shapes

Bytes are algorithmic: every operand read once, the result written once.  A weight gradient
through cdp_k_conv is three launches (clear, partial sums, fold); inside the engine the clear
does not exist and the other two are shared by all layers of a tick level.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as b

HBM_PEAK, MFMA_PEAK = 8000.0, 2500.0   # GB/s, TFLOP/s (bf16 dense)


def _time(call, reps):
    for _ in range(3):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps   # microseconds per call


def linear(M, N, K, shape, reps=200):
    A = torch.randn(M, K, device="cuda").bfloat16()
    W = torch.randn(N, K, device="cuda").bfloat16()
    C = torch.empty(M, N, device="cuda")
    us = _time(lambda: b.cdp_k_gemm(1, shape, 1, 1, A.data_ptr(), W.data_ptr(), C.data_ptr(), M, N, K, K, K), reps)
    flops, byts = 2.0 * M * N * K, 2.0 * (M * K + N * K) + 4.0 * M * N
    return us, flops / us / 1e6, byts / us / 1e3


def conv(which, B, H, W, Cin, Cout, ks, st, pad, reps=20):
    Ho, Wo = (H + 2 * pad - ks) // st + 1, (W + 2 * pad - ks) // st + 1
    x = torch.randn(B, H, W, Cin, device="cuda").bfloat16()
    w = torch.randn(Cout, ks, ks, Cin, device="cuda").bfloat16()
    wt = w.permute(3, 1, 2, 0).contiguous()
    dy = torch.randn(B, Ho, Wo, Cout, device="cuda").bfloat16()
    y = torch.empty(B, Ho, Wo, Cout, device="cuda", dtype=torch.bfloat16)
    dx = torch.empty_like(x)
    dw = torch.empty(Cout, ks, ks, Cin, device="cuda")
    ws = torch.empty(64 << 20, device="cuda", dtype=torch.float32)
    if which in (0, 3, 5):      # 3 / 4: forced onto the 256 x 256 direct-to-LDS tile, 5 / 6: onto its 128 x 128 form
        call = lambda: b.cdp_k_conv(1, which, x.data_ptr(), w.data_ptr(), y.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    elif which in (1, 4, 6):
        call = lambda: b.cdp_k_conv(1, which, dy.data_ptr(), wt.data_ptr(), dx.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
    else:
        call = lambda: b.cdp_k_conv(1, 2, dy.data_ptr(), x.data_ptr(), dw.data_ptr(), B, H, W, Cin, Cout, ks, st, pad,
                                    ws.data_ptr(), ws.numel() * 4)
    us = _time(call, reps)
    flops = 2.0 * B * Ho * Wo * Cout * ks * ks * Cin
    byts = 2.0 * (B * H * W * Cin + B * Ho * Wo * Cout) + (4 if which == 2 else 2) * Cout * ks * ks * Cin
    return us, flops / us / 1e6, byts / us / 1e3


def vit_kernels(reps=50):
    """LayerNorm, GELU and the attention core at the ViT-B/16 shapes of one micro-batch (bf16):
    (label, microseconds, algorithmic GB/s)."""
    rows, D, H, T, Bn = 6272, 768, 12, 196, 32
    bf = torch.bfloat16
    x = torch.randn(rows, D, device="cuda").to(bf)
    dy = torch.randn(rows, D, device="cuda").to(bf)
    out = torch.empty_like(x)
    gam, bet = torch.ones(D, device="cuda"), torch.zeros(D, device="cuda")
    dg, db = torch.zeros(D, device="cuda"), torch.zeros(D, device="cuda")
    ws = torch.empty(2 * rows + 2 * D * ((rows + 31) // 32) + 64, device="cuda")
    res = []
    us = _time(lambda: b.cdp_k_layernorm(1, 0, x.data_ptr(), 0, 0, gam.data_ptr(), bet.data_ptr(), out.data_ptr(), 0, 0, 0, 0,
                                         rows, D), reps)
    res.append(("layernorm fwd 6272x768", us, 2 * 2.0 * rows * D / us / 1e3))
    us = _time(lambda: b.cdp_k_layernorm(1, 1, x.data_ptr(), dy.data_ptr(), 0, gam.data_ptr(), 0, out.data_ptr(), dg.data_ptr(),
                                         db.data_ptr(), ws.data_ptr(), ws.numel() * 4, rows, D), reps)
    res.append(("layernorm bwd 6272x768 (3 kernels)", us, 5 * 2.0 * rows * D / us / 1e3))
    n = rows * 4 * D
    xg, dyg = torch.randn(n, device="cuda").to(bf), torch.randn(n, device="cuda").to(bf)
    og = torch.empty_like(xg)
    us = _time(lambda: b.cdp_k_gelu(1, 0, xg.data_ptr(), 0, og.data_ptr(), n), reps)
    res.append(("gelu fwd 6272x3072", us, 2 * 2.0 * n / us / 1e3))
    us = _time(lambda: b.cdp_k_gelu(1, 1, xg.data_ptr(), dyg.data_ptr(), og.data_ptr(), n), reps)
    res.append(("gelu bwd 6272x3072", us, 3 * 2.0 * n / us / 1e3))
    qkv = torch.randn(Bn, T, 3 * D, device="cuda").to(bf)
    do = torch.randn(Bn, T, D, device="cuda").to(bf)
    tt = Bn * H * T * T
    P = torch.empty(tt, device="cuda", dtype=bf)
    o = torch.empty(Bn, T, D, device="cuda", dtype=bf)
    dq = torch.empty_like(qkv)
    wsa = torch.empty(2 * tt + 128, device="cuda")
    us = _time(lambda: b.cdp_k_attention(1, 0, qkv.data_ptr(), P.data_ptr(), 0, o.data_ptr(), wsa.data_ptr(), wsa.numel() * 4,
                                         Bn, T, D, H), reps)
    res.append(("attention fwd 32x12 heads, 196 tokens (2 kernels)", us, 2.0 * (qkv.numel() + tt + o.numel()) / us / 1e3))
    us = _time(lambda: b.cdp_k_attention(1, 1, qkv.data_ptr(), P.data_ptr(), do.data_ptr(), dq.data_ptr(), wsa.data_ptr(),
                                         wsa.numel() * 4, Bn, T, D, H), reps)
    res.append(("attention bwd 32x12 heads, 196 tokens (4 kernels)", us, 2.0 * (2 * qkv.numel() + tt + do.numel()) / us / 1e3))
    return res


LINEAR_SHAPES = [  # (label, M, N, K, tile_shape)
    ("cfg2 layer  32x1024x1024 (thin tiles)", 32, 1024, 1024, 5),
    ("cfg2 stem   32x1024x3072 (thin tiles)", 32, 1024, 3072, 5),
    ("cfg5 layer  64x4096x4096 (64x128 tiles)", 64, 4096, 4096, 4),
    ("8 x cfg5    64x32768x4096 (64x128 tiles)", 64, 32768, 4096, 4),
]
CONV_SHAPES = [  # ResNet-50 layers of one micro-batch of 32, and two large compute-bound shapes
    ("s1 1x1 256->64  56x56", 32, 56, 56, 256, 64, 1, 1, 0), ("s1 3x3 64->64   56x56", 32, 56, 56, 64, 64, 3, 1, 1),
    ("s1 1x1 64->256  56x56", 32, 56, 56, 64, 256, 1, 1, 0), ("s2 3x3 128->128 28x28", 32, 28, 28, 128, 128, 3, 1, 1),
    ("s3 1x1 1024->256 14x14", 32, 14, 14, 1024, 256, 1, 1, 0), ("s3 3x3 256->256 14x14", 32, 14, 14, 256, 256, 3, 1, 1),
    ("s4 3x3 512->512 7x7", 32, 7, 7, 512, 512, 3, 1, 1), ("s4 1x1 512->2048 7x7", 32, 7, 7, 512, 2048, 1, 1, 0),
    ("large 1x1 2048->2048, 25088 rows", 32, 28, 28, 2048, 2048, 1, 1, 0),
    ("large 3x3 512->512, 25088 rows", 32, 28, 28, 512, 512, 3, 1, 1),
    # token-wise linear maps of a ViT-B/16-shaped block, one micro-batch of 32 x 196 tokens
    ("vit qkv 768->2304, 6272 rows", 32, 14, 14, 768, 2304, 1, 1, 0), ("vit proj 768->768, 6272 rows", 32, 14, 14, 768, 768, 1, 1, 0),
    ("vit fc1 768->3072, 6272 rows", 32, 14, 14, 768, 3072, 1, 1, 0), ("vit fc2 3072->768, 6272 rows", 32, 14, 14, 3072, 768, 1, 1, 0),
]


def main():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--only", default="", help="run only the shapes whose label contains this text")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("kernel_bench needs a GPU")
    torch.zeros(1).cuda()
    print("# Linear contractions (cdp_k_gemm, bf16): us, TFLOP/s, GB/s, fraction of the HBM peak of %.0f GB/s" % HBM_PEAK)
    for label, M, N, K, shape in LINEAR_SHAPES:
        if args.only not in label:
            continue
        us, tf, gb = linear(M, N, K, shape)
        print("%-42s %8.1f us %7.1f TFLOP/s %7.0f GB/s  hbm %.2f" % (label, us, tf, gb, gb / HBM_PEAK), flush=True)
    if args.only in "vit kernels":
        print("# Kernels of the ViT-shaped stages (bf16): us, algorithmic GB/s (inputs and outputs once), fraction of %.0f" % HBM_PEAK)
        for label, us, gb in vit_kernels():
            print("%-52s %8.1f us %7.0f GB/s  hbm %.2f" % (label, us, gb, gb / HBM_PEAK), flush=True)
    print("# Convolution passes (cdp_k_conv, bf16): us, TFLOP/s (fraction of %.0f), GB/s (fraction of %.0f)" % (MFMA_PEAK, HBM_PEAK))
    for s in CONV_SHAPES:
        if args.only not in s[0]:
            continue
        parts = []
        for which, name in ((0, "fwd"), (1, "dgrad"), (2, "wgrad")):
            us, tf, gb = conv(which, *s[1:])
            parts.append("%s %7.1f us %6.1f TF/s (%.2f) %5.0f GB/s (%.2f)" % (name, us, tf, tf / MFMA_PEAK, gb, gb / HBM_PEAK))
        print("%-34s %s" % (s[0], " | ".join(parts)), flush=True)
    print("# The same passes forced onto the direct-to-LDS kernel (cdp_k_conv which = 3 / 4: 256 x 256 tile, 5 / 6: 128 x 128), where the channel counts allow")
    for s in CONV_SHAPES + [("8192 x 8192 x 8192 product", 32, 16, 16, 8192, 8192, 1, 1, 0)]:
        if args.only not in s[0] or s[4] % 64 or s[5] % 64:
            continue
        parts = []
        for which, name in ((3, "fwd 256"), (4, "dgrad 256"), (5, "fwd 128"), (6, "dgrad 128")):
            us, tf, gb = conv(which, *s[1:])
            parts.append("%s %7.1f us %6.1f TF/s (%.2f)" % (name, us, tf, tf / MFMA_PEAK))
        print("%-34s %s" % (s[0], " | ".join(parts)), flush=True)


if __name__ == "__main__":
    main()
