"""Perturbed copies of the oracle's stage functions: yardsticks for "how far does finite precision
alone move the result" (both are models of the magnitude of rounding noise, not of any kernel).

This is test-side code, not part of the oracle: it wraps the oracle's per-layer functions
(oracle/layers.py) and is handed to the oracle's trainers through their ``stage_impl`` hook, so the
timeline, the update rule and the SGD step stay the oracle's.

Bf16Storage: round to bf16 (nearest even) where a bf16 training path stores values:
  * weight matrices (Linear, convolution) when a pass reads them; vectors (bias, gamma, beta,
    LayerNorm parameters) stay unrounded: a bf16 path keeps them in fp32;
  * every tensor a fused kernel would write to memory: the output of a layer unless the next
    layer is an element-wise follower of it (ReLU, affine, residual add, the loss head, the token
    reshape), the attention probabilities, the score gradient, dlogits;
  * the same for gradient tensors on the way back, and the micro-batch itself.
  Accumulation (inside a contraction, of the gradient sum, of the master weights) is unrounded.

Fp32Accumulation(seed): nothing is rounded, but every activation or activation gradient that a
contraction produces (Linear / convolution output, input gradient) is multiplied by
1 + 2^-24 sqrt(K) xi, xi ~ N(0, 1) independent per element, K the reduction length: the random-walk
model of a sum of K fp32 products accumulated in fp32.  (Weight gradients are left exact: a relative
error of 1e-6 there is not amplified by anything.)  At the benchmark sizes (10^7 and more ReLU arguments per run) that is enough to
flip the mask of the few arguments that lie within 1e-6 relative of zero, and one flipped mask moves
the gradients of every layer below it by a fraction of a percent: fp32 training of these networks
does not follow the fp64 trajectory to 1e-4 of the applied updates, and this stand-in says by how much.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

import cdp_workloads as wl
from oracle import layers as L

def stored(stage: Sequence[wl.Layer]) -> List[bool]:
    """stored[k+1]: tensor k+1 reaches memory (the next layer is not an element-wise follower of it)."""
    m = [True] * (len(stage) + 1)
    for k in range(len(stage) - 1):
        nxt = stage[k + 1]
        if nxt.src < 0 and nxt.kind in (wl.RELU, wl.AFFINE, wl.ADD, wl.CE_HEAD, wl.TOKENS):
            m[k + 1] = False
    return m


def _same(a):
    return a


def round_bf16(a):
    """fp32 -> bf16, round to nearest even, returned as float64 (32-bit integer arithmetic; equal to the
    oracle's round_bf16, which tests/test_parity_gates.py checks)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


class _PerVersion:
    """Quantised copy of a weight matrix, computed once per version of the matrix (the trainers
    replace a stage's arrays at every update and never write into them)."""

    def __init__(self, fn, keep=256):
        self.fn, self.keep, self.memo = fn, keep, {}

    def __call__(self, w):
        hit = self.memo.get(id(w))
        if hit is not None and hit[0] is w:
            return hit[1]
        if len(self.memo) >= self.keep:
            self.memo.clear()
        q = self.fn(w)
        self.memo[id(w)] = (w, q)
        return q


class StandIn:
    """stage_impl for oracle.cdp_oracle.train_schedule / train_equation.
    wq: applied to weight matrices when read; sq: applied to stored tensors; cn(y, K): applied to the
    result y of a contraction with reduction length K."""

    def __init__(self, wq=_same, sq=_same, cn=lambda y, K: y):
        self.wq, self.sq, self.cn = wq, sq, cn

    def prepare_input(self, x):
        return self.sq(x)

    def forward(self, stage, params, x, labels: Optional[np.ndarray] = None):
        rnd, wq, cn = self.sq, self.wq, self.cn
        lp = L.split_params(stage, params)
        keep = stored(stage)
        tensors, aux, loss = [x], [], None
        for k, layer in enumerate(stage):
            src = tensors[k if layer.src < 0 else layer.src]
            kind, p = layer.kind, layer.p
            a = None
            if kind == wl.LINEAR:
                y = cn(L.linear_fwd(src, wq(lp[k][0]), 0.0), p[0]) + lp[k][1]
            elif kind == wl.RELU:
                y = np.maximum(src, 0.0)
            elif kind == wl.CONV2D:
                y = cn(L.conv2d_fwd(src, wq(lp[k][0]), p[3], p[4]), p[0] * p[2] * p[2])
            elif kind == wl.AFFINE:
                y = L.affine_fwd(src, lp[k][0], lp[k][1])
            elif kind == wl.ADD:
                y = src + tensors[p[0]]
            elif kind == wl.MAXPOOL:
                y, a = L.maxpool_fwd(src, p[0], p[1], p[2])
            elif kind == wl.GAP:
                y = L.gap_fwd(src)
            elif kind == wl.LAYERNORM:
                y = L.layernorm_fwd(src, lp[k][0], lp[k][1])
            elif kind == wl.GELU:
                y = L.gelu_fwd(src)
            elif kind == wl.TOKENS:
                y = src.reshape(src.shape[0], 1, src.shape[1] * src.shape[2], src.shape[3])
            elif kind == wl.ATTENTION:
                a = rnd(L.attention_probs(src, p[0]))
                y = L.attention_apply(src, a, p[0])
            elif kind == wl.CE_HEAD:
                loss, a = L.ce_fwd(src, labels)
                a = rnd(a)
                y = np.zeros(())
            else:
                raise ValueError(kind)
            if keep[k + 1] and kind != wl.CE_HEAD:
                y = rnd(y)
            tensors.append(y)
            aux.append(a)
        return (loss if loss is not None else tensors[-1]), {"tensors": tensors, "aux": aux}

    def backward(self, stage, params, saved, dy):
        rnd, wq, cn = self.sq, self.wq, self.cn
        lp = L.split_params(stage, params)
        keep = stored(stage)
        tensors, aux = saved["tensors"], saved["aux"]
        dt: List[Optional[np.ndarray]] = [None] * len(tensors)

        def acc(idx, g):
            dt[idx] = g if dt[idx] is None else dt[idx] + g

        if dy is not None:
            acc(len(stage), dy)
        grads: List[List[np.ndarray]] = [[] for _ in stage]
        for k in range(len(stage) - 1, -1, -1):
            layer = stage[k]
            kind, p = layer.kind, layer.p
            si = k if layer.src < 0 else layer.src
            src = tensors[si]
            if kind == wl.CE_HEAD:
                acc(si, aux[k])
                continue
            g = dt[k + 1]
            if keep[k + 1]:
                g = rnd(g)
            if kind == wl.LINEAR:
                dx, dW, db = L.linear_bwd(src, wq(lp[k][0]), g)
                dx = cn(dx, p[1])
                grads[k] = [dW, db]
            elif kind == wl.RELU:
                dx = g * (src > 0)
            elif kind == wl.CONV2D:
                dx, dW = L.conv2d_bwd(src, wq(lp[k][0]), p[3], p[4], g)
                dx = cn(dx, p[1] * p[2] * p[2])
                grads[k] = [dW]
            elif kind == wl.AFFINE:
                dx, dg, dbeta = L.affine_bwd(src, lp[k][0], g)
                grads[k] = [dg, dbeta]
            elif kind == wl.ADD:
                dx = g
                acc(p[0], g)
            elif kind == wl.MAXPOOL:
                dx = L.maxpool_bwd(src.shape, aux[k], p[0], p[1], p[2], g)
            elif kind == wl.GAP:
                dx = L.gap_bwd(src.shape, g)
            elif kind == wl.LAYERNORM:
                dx, dg, dbeta = L.layernorm_bwd(src, lp[k][0], g)
                grads[k] = [dg, dbeta]
            elif kind == wl.GELU:
                dx = L.gelu_bwd(src, g)
            elif kind == wl.TOKENS:
                dx = g.reshape(src.shape)
            elif kind == wl.ATTENTION:
                ds = rnd(L.attention_score_grad(src, aux[k], p[0], g))
                dx = L.attention_input_grad(src, aux[k], ds, p[0], g)
            else:
                raise ValueError(kind)
            acc(si, dx)
        dx0 = dt[0]
        return (rnd(dx0) if dx0 is not None else None), [g for gl in grads for g in gl]


Bf16Storage = StandIn(wq=_PerVersion(round_bf16), sq=round_bf16)


def Fp32Accumulation(seed: int = 0) -> StandIn:
    rng = np.random.default_rng(seed)

    def cn(y, K):
        return y * (1.0 + (2.0 ** -24 * np.sqrt(float(K))) * rng.standard_normal(y.shape, dtype=np.float32))

    return StandIn(cn=cn)
