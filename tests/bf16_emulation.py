"""A perturbed copy of the oracle's stage functions that rounds to bf16 where a bf16 training
path stores values: the yardstick for "how far does bf16 storage alone move the result".

This is test-side code, not part of the oracle: it wraps the oracle's per-layer functions
(oracle/layers.py) and is handed to the oracle's trainers through their ``stage_impl`` hook, so the
timeline, the update rule and the SGD step stay the oracle's.  Rounding points (round to nearest
even, fp32 -> bf16):
  * weight matrices (Linear, convolution) when a pass reads them; vectors (bias, gamma, beta,
    LayerNorm parameters) stay unrounded: a bf16 path keeps them in fp32;
  * every tensor a fused kernel would write to memory: the output of a layer unless the next
    layer is an element-wise follower of it (ReLU, affine, residual add, the loss head, the token
    reshape), the attention probabilities, the score gradient, dlogits;
  * the same for gradient tensors on the way back, and the micro-batch itself.
Accumulation (inside a contraction, of the gradient sum, of the master weights) is unrounded.
It is a model of the magnitude of bf16 rounding noise, not of any kernel's summation order.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

import cdp_workloads as wl
from oracle import layers as L

rnd = L.round_bf16


def stored(stage: Sequence[wl.Layer]) -> List[bool]:
    """stored[k+1]: tensor k+1 reaches memory (the next layer is not an element-wise follower of it)."""
    m = [True] * (len(stage) + 1)
    for k in range(len(stage) - 1):
        nxt = stage[k + 1]
        if nxt.src < 0 and nxt.kind in (wl.RELU, wl.AFFINE, wl.ADD, wl.CE_HEAD, wl.TOKENS):
            m[k + 1] = False
    return m


class Bf16Storage:
    """stage_impl for oracle.cdp_oracle.train_schedule / train_equation."""

    @staticmethod
    def prepare_input(x):
        return rnd(x)

    @staticmethod
    def forward(stage, params, x, labels: Optional[np.ndarray] = None):
        lp = L.split_params(stage, params)
        keep = stored(stage)
        tensors, aux, loss = [x], [], None
        for k, layer in enumerate(stage):
            src = tensors[k if layer.src < 0 else layer.src]
            kind, p = layer.kind, layer.p
            a = None
            if kind == wl.LINEAR:
                y = L.linear_fwd(src, rnd(lp[k][0]), lp[k][1])
            elif kind == wl.RELU:
                y = np.maximum(src, 0.0)
            elif kind == wl.CONV2D:
                y = L.conv2d_fwd(src, rnd(lp[k][0]), p[3], p[4])
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

    @staticmethod
    def backward(stage, params, saved, dy):
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
                dx, dW, db = L.linear_bwd(src, rnd(lp[k][0]), g)
                grads[k] = [dW, db]
            elif kind == wl.RELU:
                dx = g * (src > 0)
            elif kind == wl.CONV2D:
                dx, dW = L.conv2d_bwd(src, rnd(lp[k][0]), p[3], p[4], g)
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
