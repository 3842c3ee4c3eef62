"""The entry point that allocates nothing (cdp_k_conv_wgrad_static: partial sums in a device array
that is part of the library image) against the entry point it is a variant of (cdp_k_conv, which = 2,
with a caller's workspace): same kernels, same reduction ranges, so the results must be equal bit for
bit; two calls in a row, the second on a smaller input; and both against the oracle's convolution
gradient."""
import numpy as np
import pytest

import cdp_workloads as wl
from oracle import layers as L
from paper_2403_08837_amd import binding as b

pytestmark = pytest.mark.gpu

CASES = [(4, 16, 16, 32, 64, 3, 1, 1), (2, 8, 8, 16, 32, 3, 2, 1)]   # the second is smaller in every extent


def _rnd(a, dtype):
    return L.round_bf16(a) if dtype == wl.BF16 else np.asarray(a, dtype=np.float32).astype(np.float64)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_static_scratch_weight_gradient_equals_workspace_variant(dtype):
    import torch
    assert torch.cuda.is_available()
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float32
    for n, (B, H, W, Cin, Cout, ks, st, pad) in enumerate(CASES):
        Ho, Wo = (H + 2 * pad - ks) // st + 1, (W + 2 * pad - ks) // st + 1
        x = wl.random_normal(11 + n, 1, B * H * W * Cin).reshape(B, H, W, Cin)
        dy = wl.random_normal(11 + n, 2, B * Ho * Wo * Cout).reshape(B, Ho, Wo, Cout)
        xd = torch.tensor(x, dtype=torch.float32).to(tdt).cuda()
        dyd = torch.tensor(dy, dtype=torch.float32).to(tdt).cuda()
        ws = torch.full((8 << 20,), float("nan"), dtype=torch.float32, device="cuda")
        want = torch.full((Cout, ks, ks, Cin), float("nan"), dtype=torch.float32, device="cuda")
        got = torch.full((Cout, ks, ks, Cin), float("nan"), dtype=torch.float32, device="cuda")
        b.cdp_k_conv(dtype, 2, dyd.data_ptr(), xd.data_ptr(), want.data_ptr(), B, H, W, Cin, Cout, ks, st, pad, ws.data_ptr(),
                     ws.numel() * 4)
        before = torch.cuda.memory_allocated()
        b.cdp_k_conv_wgrad_static(dtype, dyd.data_ptr(), xd.data_ptr(), got.data_ptr(), B, H, W, Cin, Cout, ks, st, pad)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got, want), (dtype, n, (got - want).abs().max().item())
        _, dw = L.conv2d_bwd(_rnd(x, dtype), np.zeros((Cout, ks, ks, Cin)), st, pad, _rnd(dy, dtype))
        err = np.abs(got.cpu().numpy().astype(np.float64) - dw).max() / np.abs(dw).max()
        assert err <= 1e-5, err     # fp32 accumulation of exactly representable products


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    # 512 x 512 channels, 3 x 3: 9.4 MB of weight gradient per reduction range, several ranges
    with pytest.raises(b.CdpError) as e:
        b.cdp_k_conv_wgrad_static(wl.F32, x.data_ptr(), x.data_ptr(), x.data_ptr(), 32, 28, 28, 512, 512, 3, 1, 1)
    assert e.value.code == b.CDP_ENOMEM and "static scratch holds" in str(e.value)
    with pytest.raises(b.CdpError) as e:     # 3 input channels: not a whole 16-byte chunk
        b.cdp_k_conv_wgrad_static(wl.F32, x.data_ptr(), x.data_ptr(), x.data_ptr(), 2, 8, 8, 3, 16, 3, 1, 1)
    assert e.value.code == b.CDP_EINVAL
