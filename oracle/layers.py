"""Layer-by-layer forward / backward definitions used by the CDP oracle.

TEST INFRASTRUCTURE ONLY (see package docstring).  Everything is plain numpy in
float64, NHWC for images, one function pair per layer kind, no fusion and no
blocking: each formula is the textbook definition of the layer and of its
vector-Jacobian product.  The paper treats a stage as an opaque differentiable
module whose forward and backward run on one micro-batch (Sec. 3.1); the layer
set here is what the benchmark configurations need.

Pins (tests/test_oracle_layers.py): finite differences in fp64 for every
layer kind and for whole stages, brute-force 7-loop convolution, 1x1 conv on
1x1 images == linear, CE closed forms.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np

import cdp_workloads as wl

Array = np.ndarray


# ---------------------------------------------------------------------------
# bf16 rounding (round-to-nearest-even on the upper 16 bits of a float32)
# ---------------------------------------------------------------------------
def round_bf16(a: Array) -> Array:
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(np.float64)


# ---------------------------------------------------------------------------
# individual layers
# ---------------------------------------------------------------------------
def linear_fwd(x: Array, W: Array, b: Array) -> Array:
    return x.reshape(x.shape[0], -1) @ W.T + b


def linear_bwd(x: Array, W: Array, dy: Array):
    x2 = x.reshape(x.shape[0], -1)
    dx = (dy @ W).reshape(x.shape)
    return dx, dy.T @ x2, dy.sum(axis=0)


def conv2d_fwd(x: Array, W: Array, stride: int, pad: int) -> Array:
    """y[b,ho,wo,o] = sum_{kh,kw,c} x[b, ho*s+kh-p, wo*s+kw-p, c] * W[o,kh,kw,c]."""
    Bn, H, Wd, C = x.shape
    O, KH, KW, _ = W.shape
    Ho = (H + 2 * pad - KH) // stride + 1
    Wo = (Wd + 2 * pad - KW) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    y = np.zeros((Bn, Ho, Wo, O), dtype=x.dtype)
    for kh in range(KH):
        for kw in range(KW):
            xs = xp[:, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride, :]
            # one matrix product per tap on contiguous copies (a strided view would take numpy's slow path)
            y += (np.ascontiguousarray(xs).reshape(-1, C) @ np.ascontiguousarray(W[:, kh, kw, :].T)).reshape(Bn, Ho, Wo, O)
    return y


def conv2d_bwd(x: Array, W: Array, stride: int, pad: int, dy: Array):
    Bn, H, Wd, C = x.shape
    O, KH, KW, _ = W.shape
    _, Ho, Wo, _ = dy.shape
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    dxp = np.zeros_like(xp)
    dW = np.zeros_like(W)
    dy2 = np.ascontiguousarray(dy).reshape(-1, O)
    for kh in range(KH):
        for kw in range(KW):
            sl = (slice(None), slice(kh, kh + stride * (Ho - 1) + 1, stride),
                  slice(kw, kw + stride * (Wo - 1) + 1, stride), slice(None))
            dW[:, kh, kw, :] = dy2.T @ np.ascontiguousarray(xp[sl]).reshape(-1, C)
            dxp[sl] += (dy2 @ np.ascontiguousarray(W[:, kh, kw, :])).reshape(Bn, Ho, Wo, C)
    dx = dxp[:, pad:pad + H, pad:pad + Wd, :]
    return dx, dW


def affine_fwd(x: Array, gamma: Array, beta: Array) -> Array:
    return x * gamma + beta


def affine_bwd(x: Array, gamma: Array, dy: Array):
    red = tuple(range(x.ndim - 1))
    return dy * gamma, (dy * x).sum(axis=red), dy.sum(axis=red)


def maxpool_fwd(x: Array, ks: int, stride: int, pad: int):
    """Max over each window; also returns the flat window index of the first maximum."""
    Bn, H, Wd, C = x.shape
    Ho = (H + 2 * pad - ks) // stride + 1
    Wo = (Wd + 2 * pad - ks) // stride + 1
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)), constant_values=-np.inf)
    best = np.full((Bn, Ho, Wo, C), -np.inf, dtype=x.dtype)
    arg = np.zeros((Bn, Ho, Wo, C), dtype=np.int64)
    for kh in range(ks):
        for kw in range(ks):
            xs = xp[:, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride, :]
            better = xs > best
            best = np.where(better, xs, best)
            arg = np.where(better, kh * ks + kw, arg)
    return best, arg


def maxpool_bwd(x_shape, arg: Array, ks: int, stride: int, pad: int, dy: Array) -> Array:
    Bn, H, Wd, C = x_shape
    _, Ho, Wo, _ = dy.shape
    dxp = np.zeros((Bn, H + 2 * pad, Wd + 2 * pad, C), dtype=dy.dtype)
    for kh in range(ks):
        for kw in range(ks):
            sl = (slice(None), slice(kh, kh + stride * (Ho - 1) + 1, stride),
                  slice(kw, kw + stride * (Wo - 1) + 1, stride), slice(None))
            dxp[sl] += np.where(arg == kh * ks + kw, dy, 0.0)
    return dxp[:, pad:pad + H, pad:pad + Wd, :]


def gap_fwd(x: Array) -> Array:
    return x.mean(axis=(1, 2))


def gap_bwd(x_shape, dy: Array) -> Array:
    Bn, H, Wd, C = x_shape
    return np.broadcast_to(dy[:, None, None, :] / (H * Wd), x_shape).copy()


LN_EPS = 1e-5


def layernorm_fwd(x: Array, gamma: Array, beta: Array) -> Array:
    """y = (x - mean) / sqrt(var + eps) * gamma + beta over the last axis (biased variance)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + LN_EPS) * gamma + beta


def layernorm_bwd(x: Array, gamma: Array, dy: Array):
    """With xh = (x - mean) * rstd and g = dy * gamma:
    dx = rstd * (g - mean(g) - xh * mean(g * xh)); dgamma = sum dy * xh; dbeta = sum dy."""
    C = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xh = (x - mu) * rstd
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xh * (g * xh).mean(axis=-1, keepdims=True))
    return dx, (dy * xh).reshape(-1, C).sum(axis=0), dy.reshape(-1, C).sum(axis=0)


def _erf(x: Array) -> Array:
    from scipy.special import erf
    return erf(x)


def gelu_fwd(x: Array) -> Array:
    """x * Phi(x) with Phi the standard normal CDF."""
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_bwd(x: Array, dy: Array) -> Array:
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    return dy * (0.5 * (1.0 + _erf(x / np.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / np.sqrt(2.0 * np.pi))


def _split_qkv(qkv: Array, heads: int):
    Bn, one, T, C3 = qkv.shape
    D = C3 // 3
    dh = D // heads
    q, k, v = (qkv[:, 0, :, i * D:(i + 1) * D].reshape(Bn, T, heads, dh).transpose(0, 2, 1, 3) for i in range(3))
    return q, k, v, dh   # each [B, heads, T, dh]


def attention_probs(qkv: Array, heads: int) -> Array:
    """P[b, h] = softmax over the keys of q k^T / sqrt(dh), per sample and head: [B, heads, T, T]."""
    q, k, v, dh = _split_qkv(qkv, heads)
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(dh)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention_apply(qkv: Array, P: Array, heads: int) -> Array:
    """out = P v per head, heads concatenated along the channel axis: [B, 1, T, D]."""
    q, k, v, dh = _split_qkv(qkv, heads)
    o = P @ v                                             # [B, heads, T, dh]
    Bn, _, T, _ = o.shape
    return o.transpose(0, 2, 1, 3).reshape(Bn, 1, T, heads * dh)


def attention_fwd(qkv: Array, heads: int):
    """Per head: P = softmax(q k^T / sqrt(dh)) over the keys, out = P v.  Returns (out, P);
    P is what the backward pass keeps."""
    P = attention_probs(qkv, heads)
    return attention_apply(qkv, P, heads), P


def attention_score_grad(qkv: Array, P: Array, heads: int, dout: Array) -> Array:
    """ds = P * (dP - rowsum(dP * P)) / sqrt(dh) with dP = do v^T: gradient of the scaled scores."""
    q, k, v, dh = _split_qkv(qkv, heads)
    Bn, _, T, D = dout.shape
    do = dout[:, 0].reshape(Bn, T, heads, dh).transpose(0, 2, 1, 3)
    dP = do @ v.transpose(0, 1, 3, 2)
    return P * (dP - (dP * P).sum(axis=-1, keepdims=True)) / np.sqrt(dh)


def attention_input_grad(qkv: Array, P: Array, ds: Array, heads: int, dout: Array) -> Array:
    """dq = ds k; dk = ds^T q; dv = P^T do, laid out like qkv."""
    q, k, v, dh = _split_qkv(qkv, heads)
    Bn, _, T, D = dout.shape
    do = dout[:, 0].reshape(Bn, T, heads, dh).transpose(0, 2, 1, 3)
    dv = P.transpose(0, 1, 3, 2) @ do
    dq = ds @ k
    dk = ds.transpose(0, 1, 3, 2) @ q
    parts = [t.transpose(0, 2, 1, 3).reshape(Bn, T, D) for t in (dq, dk, dv)]
    return np.concatenate(parts, axis=-1)[:, None, :, :]


def attention_bwd(qkv: Array, P: Array, heads: int, dout: Array) -> Array:
    """dv = P^T do; dP = do v^T; ds = P * (dP - rowsum(dP * P)) / sqrt(dh); dq = ds k; dk = ds^T q."""
    return attention_input_grad(qkv, P, attention_score_grad(qkv, P, heads, dout), heads, dout)


def ce_fwd(logits: Array, labels: Array):
    """loss = mean_b [ logsumexp(z_b) - z_b[y_b] ];  dz = (softmax(z) - onehot(y)) / B."""
    Bn = logits.shape[0]
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    s = e.sum(axis=1, keepdims=True)
    lse = (m + np.log(s))[:, 0]
    loss = float((lse - logits[np.arange(Bn), labels]).mean())
    dz = e / s
    dz[np.arange(Bn), labels] -= 1.0
    return loss, dz / Bn


# ---------------------------------------------------------------------------
# stages: a list of layers over numbered tensors (tensor 0 = stage input)
# ---------------------------------------------------------------------------
def split_params(stage: Sequence[wl.Layer], params: Sequence[Array]) -> List[List[Array]]:
    out, k = [], 0
    for layer in stage:
        n = len(wl.layer_param_shapes(layer))
        out.append(list(params[k:k + n]))
        k += n
    assert k == len(params)
    return out


def stage_forward(stage: Sequence[wl.Layer], params: Sequence[Array], x: Array,
                  labels: Optional[Array] = None):
    """Run every layer in order.  Returns (output, saved) where output is the last
    tensor, or the scalar loss if the stage ends in a CE head; ``saved`` holds what
    the backward pass needs."""
    lp = split_params(stage, params)
    tensors: List[Array] = [x]
    aux: List[object] = []
    loss = None
    for k, layer in enumerate(stage):
        src = tensors[k if layer.src < 0 else layer.src]
        kind, p = layer.kind, layer.p
        a = None
        if kind == wl.LINEAR:
            y = linear_fwd(src, lp[k][0], lp[k][1])
        elif kind == wl.RELU:
            y = np.maximum(src, 0.0)
        elif kind == wl.CONV2D:
            y = conv2d_fwd(src, lp[k][0], p[3], p[4])
        elif kind == wl.AFFINE:
            y = affine_fwd(src, lp[k][0], lp[k][1])
        elif kind == wl.ADD:
            y = src + tensors[p[0]]
        elif kind == wl.MAXPOOL:
            y, a = maxpool_fwd(src, p[0], p[1], p[2])
        elif kind == wl.GAP:
            y = gap_fwd(src)
        elif kind == wl.LAYERNORM:
            y = layernorm_fwd(src, lp[k][0], lp[k][1])
        elif kind == wl.GELU:
            y = gelu_fwd(src)
        elif kind == wl.TOKENS:
            y = src.reshape(src.shape[0], 1, src.shape[1] * src.shape[2], src.shape[3])
        elif kind == wl.ATTENTION:
            y, a = attention_fwd(src, p[0])
        elif kind == wl.CE_HEAD:
            assert labels is not None and k == len(stage) - 1
            loss, a = ce_fwd(src, labels)
            y = np.zeros(())
        else:
            raise ValueError(kind)
        tensors.append(y)
        aux.append(a)
    saved = {"tensors": tensors, "aux": aux}
    return (loss if loss is not None else tensors[-1]), saved


def stage_backward(stage: Sequence[wl.Layer], params: Sequence[Array], saved, dy: Optional[Array]):
    """Vector-Jacobian product of the whole stage.  ``dy`` is the gradient of the
    micro-batch objective with respect to the stage output (None for a stage that
    ends in the CE head).  Returns (dx, grads) with grads ordered like params."""
    lp = split_params(stage, params)
    tensors, aux = saved["tensors"], saved["aux"]
    dt: List[Optional[Array]] = [None] * len(tensors)

    def acc(idx: int, g: Array) -> None:
        dt[idx] = g if dt[idx] is None else dt[idx] + g

    if dy is not None:
        acc(len(stage), dy)
    grads: List[List[Array]] = [[] for _ in stage]
    for k in range(len(stage) - 1, -1, -1):
        layer = stage[k]
        kind, p = layer.kind, layer.p
        si = k if layer.src < 0 else layer.src
        src = tensors[si]
        if kind == wl.CE_HEAD:
            acc(si, aux[k])
            continue
        g = dt[k + 1]
        assert g is not None, "tensor %d has no consumer" % (k + 1)
        if kind == wl.LINEAR:
            dx, dW, db = linear_bwd(src, lp[k][0], g)
            grads[k] = [dW, db]
        elif kind == wl.RELU:
            dx = g * (src > 0)
        elif kind == wl.CONV2D:
            dx, dW = conv2d_bwd(src, lp[k][0], p[3], p[4], g)
            grads[k] = [dW]
        elif kind == wl.AFFINE:
            dx, dg, dbeta = affine_bwd(src, lp[k][0], g)
            grads[k] = [dg, dbeta]
        elif kind == wl.ADD:
            dx = g
            acc(p[0], g)
        elif kind == wl.MAXPOOL:
            dx = maxpool_bwd(src.shape, aux[k], p[0], p[1], p[2], g)
        elif kind == wl.GAP:
            dx = gap_bwd(src.shape, g)
        elif kind == wl.LAYERNORM:
            dx, dg, dbeta = layernorm_bwd(src, lp[k][0], g)
            grads[k] = [dg, dbeta]
        elif kind == wl.GELU:
            dx = gelu_bwd(src, g)
        elif kind == wl.TOKENS:
            dx = g.reshape(src.shape)
        elif kind == wl.ATTENTION:
            dx = attention_bwd(src, aux[k], p[0], g)
        else:
            raise ValueError(kind)
        acc(si, dx)
    flat = [g for gl in grads for g in gl]
    return dt[0], flat


def model_forward_backward(stages, params_per_stage, x, labels, stage_impl=None):
    """Ordinary whole-network forward and backward on one micro-batch, each stage
    j evaluated at params_per_stage[j].  Returns (loss, grads per stage).
    ``stage_impl`` (tests only): an object whose prepare_input / forward / backward replace
    the identity, stage_forward and stage_backward of this module."""
    fwd = stage_forward if stage_impl is None else stage_impl.forward
    bwd = stage_backward if stage_impl is None else stage_impl.backward
    saved = []
    h = x if stage_impl is None else stage_impl.prepare_input(x)
    for j, st in enumerate(stages):
        h, sv = fwd(st, params_per_stage[j], h, labels if j == len(stages) - 1 else None)
        saved.append(sv)
    loss = h
    grads = [None] * len(stages)
    dy = None
    for j in range(len(stages) - 1, -1, -1):
        dy, grads[j] = bwd(stages[j], params_per_stage[j], saved[j], dy)
    return loss, grads
