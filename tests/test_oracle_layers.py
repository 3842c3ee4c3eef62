"""Pins of the oracle's layer definitions: finite differences, brute force, closed forms,
and PyTorch's CPU autograd as an independent library routine.  No GPU."""
import math

import numpy as np
import pytest
import torch

import cdp_workloads as wl
from oracle import layers as L


def _rand(shape, seed):
    return wl.random_normal(7, seed, int(np.prod(shape))).reshape(shape)


def _fd_check(f, x, dx_analytic, n=40, seed=0, tol=1e-6):
    """Central differences of scalar f at x along sampled coordinates.  A ReLU or max
    kink inside [x-h, x+h] spoils a difference quotient, so a coordinate passes if the
    quotient agrees for one of three step sizes."""
    rs = np.random.RandomState(seed)
    flat = x.ravel()
    scale = max(1e-12, float(np.abs(dx_analytic).max()))
    for _ in range(min(n, flat.size)):
        k = rs.randint(flat.size)
        old = flat[k]
        errs = []
        for h, t in ((1e-5, tol), (1e-6, 10 * tol), (1e-7, 100 * tol)):
            flat[k] = old + h
            fp = f()
            flat[k] = old - h
            fm = f()
            flat[k] = old
            errs.append(abs((fp - fm) / (2 * h) - dx_analytic.ravel()[k]) / (t * scale + 1e-9))
            if errs[-1] <= 1.0:
                break
        assert min(errs) <= 1.0, (k, errs, dx_analytic.ravel()[k])


# --- closed forms -----------------------------------------------------------------
@pytest.mark.parametrize("C", [10, 1000])
def test_ce_zero_logits_is_log_c(C):
    loss, dz = L.ce_fwd(np.zeros((4, C)), np.array([0, 1, 2, 3]))
    assert abs(loss - math.log(C)) < 1e-12
    assert abs(math.log(10) - 2.302585) < 1e-6 and abs(math.log(1000) - 6.907755) < 1e-6
    assert np.abs(dz.sum(axis=1)).max() < 1e-15
    assert abs(dz[0, 0] - (1.0 / C - 1.0) / 4) < 1e-15 and abs(dz[0, 1] - (1.0 / C) / 4) < 1e-15


def test_ce_shift_invariance_and_large_logits():
    z = _rand((5, 7), 1) * 30
    y = np.array([0, 6, 3, 3, 1])
    l0, d0 = L.ce_fwd(z, y)
    l1, d1 = L.ce_fwd(z + 1000.0, y)
    assert abs(l0 - l1) < 1e-9 and np.abs(d0 - d1).max() < 1e-12
    assert np.isfinite(l1)


def test_bf16_rounding_known_values():
    # 1 + 2^-8 is a tie between 1 and 1+2^-7: round to even -> 1; 1 + 3*2^-8 ties to 1+2^-6
    v = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 3.0e38])
    r = L.round_bf16(v)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -7 and r[3] == 1.0 + 2 ** -6 and r[4] == -2.5
    t = torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(r, t)
    x = _rand((4096,), 3)
    assert np.array_equal(L.round_bf16(x), torch.tensor(x, dtype=torch.float32).bfloat16().double().numpy())


# --- convolution: brute force, linear special case --------------------------------
@pytest.mark.parametrize("ks,stride,pad,H,W", [(3, 1, 1, 5, 6), (3, 2, 1, 7, 5), (1, 2, 0, 6, 6), (7, 2, 3, 12, 9)])
def test_conv_matches_seven_loops(ks, stride, pad, H, W):
    B, C, Oc = 2, 3, 4
    x, Wt = _rand((B, H, W, C), 1), _rand((Oc, ks, ks, C), 2)
    y = L.conv2d_fwd(x, Wt, stride, pad)
    Ho, Wo = (H + 2 * pad - ks) // stride + 1, (W + 2 * pad - ks) // stride + 1
    ref = np.zeros((B, Ho, Wo, Oc))
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for o in range(Oc):
                    for kh in range(ks):
                        for kw in range(ks):
                            for c in range(C):
                                hi, wi = ho * stride + kh - pad, wo * stride + kw - pad
                                if 0 <= hi < H and 0 <= wi < W:
                                    ref[b, ho, wo, o] += x[b, hi, wi, c] * Wt[o, kh, kw, c]
    assert y.shape == ref.shape and np.abs(y - ref).max() < 1e-12
    # backward against brute-force adjoints
    dy = _rand(y.shape, 3)
    dx, dW = L.conv2d_bwd(x, Wt, stride, pad, dy)
    rdx, rdW = np.zeros_like(x), np.zeros_like(Wt)
    for b in range(B):
        for ho in range(Ho):
            for wo in range(Wo):
                for o in range(Oc):
                    for kh in range(ks):
                        for kw in range(ks):
                            hi, wi = ho * stride + kh - pad, wo * stride + kw - pad
                            if 0 <= hi < H and 0 <= wi < W:
                                rdx[b, hi, wi, :] += dy[b, ho, wo, o] * Wt[o, kh, kw, :]
                                rdW[o, kh, kw, :] += dy[b, ho, wo, o] * x[b, hi, wi, :]
    assert np.abs(dx - rdx).max() < 1e-12 and np.abs(dW - rdW).max() < 1e-12


def test_conv_1x1_on_1x1_is_linear():
    x, Wt = _rand((5, 1, 1, 6), 1), _rand((4, 1, 1, 6), 2)
    y = L.conv2d_fwd(x, Wt, 1, 0)
    assert np.abs(y[:, 0, 0, :] - L.linear_fwd(x[:, 0, 0, :], Wt[:, 0, 0, :], np.zeros(4))).max() < 1e-13


def test_conv_and_pool_match_torch():
    x, Wt = _rand((2, 9, 8, 3), 1), _rand((5, 3, 3, 3), 2)
    xt = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(Wt).permute(0, 3, 1, 2).requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=2, padding=1)
    y = L.conv2d_fwd(x, Wt, 2, 1)
    assert np.abs(yt.detach().permute(0, 2, 3, 1).numpy() - y).max() < 1e-12
    dy = _rand(y.shape, 3)
    yt.backward(torch.tensor(dy).permute(0, 3, 1, 2))
    dx, dW = L.conv2d_bwd(x, Wt, 2, 1, dy)
    assert np.abs(xt.grad.permute(0, 2, 3, 1).numpy() - dx).max() < 1e-12
    assert np.abs(wt.grad.permute(0, 2, 3, 1).numpy() - dW).max() < 1e-12
    # max pool 3x3/2 pad 1
    xp = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    pt = torch.nn.functional.max_pool2d(xp, 3, 2, 1)
    p, arg = L.maxpool_fwd(x, 3, 2, 1)
    assert np.array_equal(pt.detach().permute(0, 2, 3, 1).numpy(), p)
    dp = _rand(p.shape, 4)
    pt.backward(torch.tensor(dp).permute(0, 3, 1, 2))
    assert np.abs(xp.grad.permute(0, 2, 3, 1).numpy() - L.maxpool_bwd(x.shape, arg, 3, 2, 1, dp)).max() < 1e-13


# --- finite differences: every layer kind through whole stages ----------------------
def _stage_fd(stage, in_shape, labels=None, seed=0):
    B = 3
    x = _rand((B,) + in_shape, 10 + seed)
    params = []
    for k, shp in enumerate(wl.stage_param_shapes(stage)):
        params.append(_rand(shp, 20 + k + seed) * 0.5 + (1.0 if len(shp) == 1 else 0.0))
    out_shape = wl.stage_tensor_shapes(stage, in_shape)[-1]
    has_head = stage[-1].kind == wl.CE_HEAD
    proj = None if has_head else _rand((B,) + out_shape, 30 + seed)

    def f():
        out, _ = L.stage_forward(stage, params, x, labels)
        return float(out) if has_head else float((out * proj).sum())

    _, saved = L.stage_forward(stage, params, x, labels)
    dx, grads = L.stage_backward(stage, params, saved, None if has_head else proj)
    _fd_check(f, x, dx)
    for p, g in zip(params, grads):
        assert p.shape == g.shape
        _fd_check(f, p, g)


def test_fd_linear_relu_stage():
    _stage_fd([wl.Layer(wl.LINEAR, (6, 5)), wl.Layer(wl.RELU)], (6,))


def test_fd_head_stage():
    st = [wl.Layer(wl.LINEAR, (6, 5)), wl.Layer(wl.RELU), wl.Layer(wl.LINEAR, (5, 4)), wl.Layer(wl.CE_HEAD, (4,))]
    _stage_fd(st, (6,), labels=np.array([0, 3, 1]))


def test_fd_basic_block_with_projection_and_stem():
    cfg = wl.get_config("resnet18_mini")
    shapes = wl.config_stage_in_shapes(cfg)
    _stage_fd(cfg.stages[0], shapes[0])          # stem + identity-shortcut block
    _stage_fd(cfg.stages[2], shapes[2], seed=1)  # stride-2 block with 1x1 projection shortcut


def test_fd_last_stage_gap_fc_ce():
    cfg = wl.get_config("resnet18_mini")
    shapes = wl.config_stage_in_shapes(cfg)
    _stage_fd(cfg.stages[-1], (2, 2, 64) if False else shapes[-1], labels=np.array([1, 9, 4]))


def test_fd_bottleneck_stem_with_maxpool():
    cfg = wl.get_config("resnet50_mini")
    st = cfg.stages[0]
    assert any(l.kind == wl.MAXPOOL for l in st)
    _stage_fd(st, (12, 12, 3))
    shapes = wl.config_stage_in_shapes(cfg)
    _stage_fd(cfg.stages[3], shapes[3], seed=2)  # stride-2 bottleneck with projection


# --- torch autograd on whole networks -------------------------------------------------
def torch_forward(stages, params, x, y):
    """The same network written with torch.nn.functional (NCHW), for autograd pins."""
    import torch.nn.functional as F
    h = x
    for st, plist in zip(stages, params):
        tensors = [h]
        k = 0
        for li, layer in enumerate(st):
            src = tensors[li if layer.src < 0 else layer.src]
            if layer.kind == wl.LINEAR:
                out = F.linear(src.reshape(src.shape[0], -1), plist[k], plist[k + 1]); k += 2
            elif layer.kind == wl.RELU:
                out = torch.relu(src)
            elif layer.kind == wl.CONV2D:
                out = F.conv2d(src, plist[k].permute(0, 3, 1, 2), stride=layer.p[3], padding=layer.p[4]); k += 1
            elif layer.kind == wl.AFFINE:
                out = src * plist[k].view(1, -1, 1, 1) + plist[k + 1].view(1, -1, 1, 1); k += 2
            elif layer.kind == wl.ADD:
                out = src + tensors[layer.p[0]]
            elif layer.kind == wl.MAXPOOL:
                out = F.max_pool2d(src, layer.p[0], layer.p[1], layer.p[2])
            elif layer.kind == wl.GAP:
                out = src.mean(dim=(2, 3))
            elif layer.kind == wl.LAYERNORM:      # channels are dim 1 in NCHW
                out = F.layer_norm(src.permute(0, 2, 3, 1), (layer.p[0],), plist[k], plist[k + 1], eps=1e-5).permute(0, 3, 1, 2); k += 2
            elif layer.kind == wl.GELU:
                out = F.gelu(src)
            elif layer.kind == wl.TOKENS:
                out = src.reshape(src.shape[0], src.shape[1], 1, src.shape[2] * src.shape[3])
            elif layer.kind == wl.ATTENTION:
                Bn, C3, _, T = src.shape
                heads, D = layer.p[0], C3 // 3
                tok = src[:, :, 0, :].permute(0, 2, 1)                       # [B, T, 3D]
                q, kk, v = (tok[:, :, i * D:(i + 1) * D].reshape(Bn, T, heads, D // heads).transpose(1, 2) for i in range(3))
                o = F.scaled_dot_product_attention(q, kk, v)                  # [B, heads, T, dh]
                out = o.transpose(1, 2).reshape(Bn, T, D).permute(0, 2, 1)[:, :, None, :]
            elif layer.kind == wl.CE_HEAD:
                out = F.cross_entropy(src, y, reduction="mean")
            tensors.append(out)
        h = tensors[-1]
    return h


def to_torch_params(params):
    return [[torch.tensor(np.asarray(p, dtype=np.float64), requires_grad=True) for p in st] for st in params]


def to_torch_x(x):
    t = torch.tensor(np.asarray(x, dtype=np.float64))
    return t.permute(0, 3, 1, 2) if t.dim() == 4 else t


@pytest.mark.parametrize("name", ["mlp_odd", "resnet18_mini", "resnet50_mini", "vit_mini"])
def test_whole_network_gradient_matches_torch_autograd(name):
    cfg = wl.get_config(name)
    params = wl.init_params(cfg, seed=3)
    # perturb zero biases / unit gammas so every parameter matters
    params = [[p + 0.1 * _rand(p.shape, 50 + k).astype(np.float32) for k, p in enumerate(st)] for st in params]
    x, y = wl.make_batch(cfg, 0, seed=3)
    x, y = x[:cfg.B], y[:cfg.B]
    p64 = [[np.asarray(p, dtype=np.float64) for p in st] for st in params]
    loss, grads = L.model_forward_backward(cfg.stages, p64, np.asarray(x, dtype=np.float64), y)
    tp = to_torch_params(params)
    tl = torch_forward(cfg.stages, tp, to_torch_x(x), torch.tensor(y, dtype=torch.long))
    tl.backward()
    assert abs(float(tl) - loss) < 1e-10 * max(1.0, abs(loss))
    for gs, ts in zip(grads, tp):
        for g, t in zip(gs, ts):
            ref = t.grad.numpy()
            assert np.abs(g - ref).max() <= 1e-10 * max(1e-3, np.abs(ref).max())


# --- transformer layers -----------------------------------------------------------
def test_layernorm_closed_forms_and_fd():
    x = _rand((3, 1, 5, 12), 1) * 2.0 + 0.7
    g, bta = 1.0 + 0.3 * _rand((12,), 2), 0.2 * _rand((12,), 3)
    y = L.layernorm_fwd(x, np.ones(12), np.zeros(12))
    assert np.abs(y.mean(axis=-1)).max() < 1e-12                       # zero mean per position
    assert np.abs((y ** 2).mean(axis=-1) - 1.0).max() < 1e-4           # unit variance up to eps
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (12,), torch.tensor(g), torch.tensor(bta), eps=1e-5).numpy()
    assert np.abs(L.layernorm_fwd(x, g, bta) - ref).max() < 1e-12
    w = _rand(x.shape, 4)
    dx, dg, db = L.layernorm_bwd(x, g, w)
    _fd_check(lambda: float((L.layernorm_fwd(x, g, bta) * w).sum()), x, dx)
    _fd_check(lambda: float((L.layernorm_fwd(x, g, bta) * w).sum()), g, dg)
    _fd_check(lambda: float((L.layernorm_fwd(x, g, bta) * w).sum()), bta, db)
    assert np.abs(dx.sum(axis=-1)).max() < 1e-10                       # shifts of a position's input do not matter


def test_gelu_closed_forms_and_fd():
    assert L.gelu_fwd(np.zeros(1))[0] == 0.0
    assert abs(L.gelu_bwd(np.zeros(1), np.ones(1))[0] - 0.5) < 1e-15
    x = _rand((4, 7), 5) * 2.0
    assert np.abs(L.gelu_fwd(x) - torch.nn.functional.gelu(torch.tensor(x)).numpy()).max() < 1e-12
    assert np.abs(L.gelu_fwd(np.array([20.0, -20.0])) - np.array([20.0, 0.0])).max() < 1e-12
    w = _rand(x.shape, 6)
    _fd_check(lambda: float((L.gelu_fwd(x) * w).sum()), x, L.gelu_bwd(x, w))


def test_attention_definition_library_and_fd():
    Bn, T, heads, dh = 2, 5, 3, 4
    D = heads * dh
    qkv = _rand((Bn, 1, T, 3 * D), 7)
    out, P = L.attention_fwd(qkv, heads)
    assert np.abs(P.sum(axis=-1) - 1.0).max() < 1e-12 and (P > 0).all()
    # brute force from the definition, one (sample, head, query) at a time
    for b in range(Bn):
        for h in range(heads):
            q = qkv[b, 0, :, h * dh:(h + 1) * dh]
            k = qkv[b, 0, :, D + h * dh:D + (h + 1) * dh]
            v = qkv[b, 0, :, 2 * D + h * dh:2 * D + (h + 1) * dh]
            for t in range(T):
                sc = np.array([q[t] @ k[u] for u in range(T)]) / math.sqrt(dh)
                p = np.exp(sc - sc.max()); p /= p.sum()
                assert np.abs(sum(p[u] * v[u] for u in range(T)) - out[b, 0, t, h * dh:(h + 1) * dh]).max() < 1e-12
    # identical keys: uniform attention, the output is the mean value
    same = qkv.copy()
    same[:, :, :, D:2 * D] = same[:, :, :1, D:2 * D]
    o2, P2 = L.attention_fwd(same, heads)
    assert np.abs(P2 - 1.0 / T).max() < 1e-12
    assert np.abs(o2 - same[:, :, :, 2 * D:].mean(axis=2, keepdims=True)).max() < 1e-12
    w = _rand(out.shape, 8)
    dqkv = L.attention_bwd(qkv, P, heads, w)
    _fd_check(lambda: float((L.attention_fwd(qkv, heads)[0] * w).sum()), qkv, dqkv)


def test_fd_transformer_block_stage():
    cfg = wl.get_config("vit_mini")
    _stage_fd(cfg.stages[1], (1, 16, 32), seed=3)
    _stage_fd(cfg.stages[0], (16, 16, 3), seed=4)
    _stage_fd(cfg.stages[3], (1, 16, 32), labels=np.array([1, 0, 7]), seed=5)
