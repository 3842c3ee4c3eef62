"""ctypes binding of libcdp (include/cdp.h): argument marshalling only.

Every step of the CDP hot path runs inside the library's HIP kernels; PyTorch is used
by callers only to own device memory (the arena, inputs) and the stream.  There is no
CPU fallback: loading fails loudly when libcdp.so has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcdp.so")

CDP_OK, CDP_EINVAL, CDP_ENOMEM, CDP_ESTATE, CDP_EHIP = 0, -1, -2, -3, -4
CDP_RULE_DP, CDP_RULE_V1, CDP_RULE_V2 = 0, 1, 2
CDP_F32, CDP_BF16 = 0, 1

EXPORTS = ["cdp_arena_bytes", "cdp_init", "cdp_set_weights", "cdp_param_count", "cdp_tick", "cdp_step",
           "cdp_drain", "cdp_get_weights", "cdp_get_losses", "cdp_get_trace", "cdp_get_live_counts",
           "cdp_get_live_bytes", "cdp_get_stats", "cdp_last_error", "cdp_destroy", "cdp_profile_gemm", "cdp_get_gemm_profile",
           "cdp_k_gemm", "cdp_k_conv", "cdp_k_conv_wgrad_static", "cdp_k_layernorm", "cdp_k_gelu", "cdp_k_attention"]


class cdp_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("src", C.c_int32), ("p", C.c_int32 * 6)]


class cdp_stage_desc(C.Structure):
    _fields_ = [("layers", C.POINTER(cdp_layer_desc)), ("n_layers", C.c_int32)]


class cdp_opts(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("dry_run", C.c_int32), ("in_rank", C.c_int32), ("in_dims", C.c_int32 * 3),
                ("hip_stream", C.c_void_p), ("arena", C.c_void_p), ("arena_bytes", C.c_size_t),
                ("momentum", C.c_float), ("weight_decay", C.c_float), ("dp_batched", C.c_int32),
                ("fresh_mask", C.c_void_p), ("bwd_fresh", C.c_int32), ("dw_group", C.c_int32)]


class cdp_trace_rec(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("tick", "mb", "step", "stage", "dir", "version")]


class cdp_stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "ticks_run", "steps_enqueued", "peak_live_stage_inputs", "last_live_stage_inputs", "peak_activation_bytes",
        "cur_activation_bytes", "pool_span_bytes", "dp_activation_bytes", "weight_bytes", "kernel_launches",
        "scratch_bytes")]


class cdp_gemm_profile(C.Structure):
    _fields_ = [("launches", C.c_int64), ("total_ms", C.c_double), ("flops", C.c_double), ("bytes", C.c_double),
                ("empty_pair_ms", C.c_double)]


class CdpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libcdp error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libcdp.so is not built: run `python -m paper_2403_08837_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
        L.cdp_arena_bytes.argtypes = [C.POINTER(cdp_stage_desc), i32, i32, i32, i32, C.POINTER(cdp_opts), C.POINTER(sz)]
        L.cdp_init.argtypes = [C.POINTER(vp), C.POINTER(cdp_stage_desc), i32, i32, i32, C.c_float, i32, C.POINTER(cdp_opts)]
        L.cdp_set_weights.argtypes = [vp, i32, C.POINTER(C.c_float), sz]
        L.cdp_param_count.argtypes = [vp, i32, C.POINTER(sz)]
        L.cdp_tick.argtypes = [vp, vp, vp]
        L.cdp_step.argtypes = [vp, vp, vp]
        L.cdp_drain.argtypes = [vp]
        L.cdp_get_weights.argtypes = [vp, i32, i32, C.POINTER(C.c_float), sz, C.POINTER(sz)]
        L.cdp_get_losses.argtypes = [vp, C.c_int64, C.POINTER(C.c_float), sz]
        L.cdp_get_trace.argtypes = [vp, C.POINTER(cdp_trace_rec), sz, C.POINTER(sz)]
        L.cdp_get_live_counts.argtypes = [vp, C.POINTER(C.c_int32), sz, C.POINTER(sz)]
        L.cdp_get_live_bytes.argtypes = [vp, i32, C.POINTER(C.c_int64), sz, C.POINTER(sz)]
        L.cdp_get_stats.argtypes = [vp, C.POINTER(cdp_stats)]
        L.cdp_last_error.argtypes = [vp]
        L.cdp_last_error.restype = C.c_char_p
        L.cdp_destroy.argtypes = [vp]
        L.cdp_destroy.restype = None
        L.cdp_profile_gemm.argtypes = [vp, i32]
        L.cdp_get_gemm_profile.argtypes = [vp, C.POINTER(cdp_gemm_profile)]
        L.cdp_k_gemm.argtypes = [i32, i32, i32, i32, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.cdp_k_conv.argtypes = [i32, i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        L.cdp_k_conv_wgrad_static.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.cdp_k_layernorm.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, i32, i32, vp]
        L.cdp_k_gelu.argtypes = [i32, i32, vp, vp, vp, C.c_int64, vp]
        L.cdp_k_attention.argtypes = [i32, i32, vp, vp, vp, vp, vp, sz, i32, i32, i32, i32, vp]
        for name in EXPORTS:
            if name not in ("cdp_last_error", "cdp_destroy"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int, ctx=None) -> None:
    if rc != CDP_OK:
        raise CdpError(rc, lib().cdp_last_error(ctx).decode())


def marshal_stages(stages: Sequence[Sequence[object]]):
    """stages: per stage a sequence of objects with .kind, .src, .p (cdp_workloads.Layer)."""
    keep = []
    arr = (cdp_stage_desc * len(stages))()
    for s, layers in enumerate(stages):
        la = (cdp_layer_desc * len(layers))()
        for k, l in enumerate(layers):
            la[k].kind, la[k].src = int(l.kind), int(l.src)
            for q, v in enumerate(l.p):
                la[k].p[q] = int(v)
        keep.append(la)
        arr[s].layers = C.cast(la, C.POINTER(cdp_layer_desc))
        arr[s].n_layers = len(layers)
    return arr, keep


def make_opts(dtype: int, in_shape: Sequence[int], dry_run: bool = False, stream: int = 0, arena: int = 0,
              arena_bytes: int = 0, momentum: float = 0.0, weight_decay: float = 0.0,
              dp_batched: bool = False, fresh_mask=None, bwd_fresh: bool = False, dw_group: int = 1) -> cdp_opts:
    o = cdp_opts()
    o.dtype, o.dry_run, o.in_rank = int(dtype), int(bool(dry_run)), len(in_shape)
    for k, v in enumerate(in_shape):
        o.in_dims[k] = int(v)
    o.hip_stream, o.arena, o.arena_bytes = stream or None, arena or None, int(arena_bytes)
    o.momentum, o.weight_decay = float(momentum), float(weight_decay)
    o.dp_batched = int(bool(dp_batched))
    o.bwd_fresh = int(bool(bwd_fresh))
    o.dw_group = int(dw_group)
    if fresh_mask is not None:
        m = np.ascontiguousarray(np.asarray(fresh_mask) != 0, dtype=np.uint8)
        o._mask_keepalive = m           # the library copies it during cdp_init
        o.fresh_mask = m.ctypes.data
    else:
        o.fresh_mask = None
    return o


# ---- functions named like the C ABI --------------------------------------------------
def cdp_arena_bytes(stages, N: int, B: int, rule: int, opts: cdp_opts) -> int:
    arr, _keep = marshal_stages(stages)
    out = C.c_size_t(0)
    _check(lib().cdp_arena_bytes(arr, len(stages), N, B, rule, C.byref(opts), C.byref(out)))
    return int(out.value)


def cdp_init(stages, N: int, B: int, lr: float, rule: int, opts: cdp_opts) -> C.c_void_p:
    arr, _keep = marshal_stages(stages)
    ctx = C.c_void_p()
    _check(lib().cdp_init(C.byref(ctx), arr, len(stages), N, B, float(lr), rule, C.byref(opts)))
    return ctx


def cdp_param_count(ctx, stage: int) -> int:
    n = C.c_size_t(0)
    _check(lib().cdp_param_count(ctx, stage, C.byref(n)), ctx)
    return int(n.value)


def cdp_set_weights(ctx, stage: int, flat: np.ndarray) -> None:
    a = np.ascontiguousarray(flat, dtype=np.float32)
    _check(lib().cdp_set_weights(ctx, stage, a.ctypes.data_as(C.POINTER(C.c_float)), a.size), ctx)


def cdp_tick(ctx, x_ptr: int, y_ptr: int) -> None:
    _check(lib().cdp_tick(ctx, x_ptr or None, y_ptr or None), ctx)


def cdp_step(ctx, x_ptr: int, y_ptr: int) -> None:
    _check(lib().cdp_step(ctx, x_ptr, y_ptr), ctx)


def cdp_drain(ctx) -> None:
    _check(lib().cdp_drain(ctx), ctx)


def cdp_get_weights(ctx, stage: int, version: int = -1) -> np.ndarray:
    n = cdp_param_count(ctx, stage)
    out = np.empty(n, dtype=np.float32)
    got = C.c_size_t(0)
    _check(lib().cdp_get_weights(ctx, stage, version, out.ctypes.data_as(C.POINTER(C.c_float)), n, C.byref(got)), ctx)
    return out


def cdp_get_losses(ctx, step: int, N: int) -> np.ndarray:
    out = np.empty(N, dtype=np.float32)
    _check(lib().cdp_get_losses(ctx, step, out.ctypes.data_as(C.POINTER(C.c_float)), N), ctx)
    return out


def cdp_get_trace(ctx) -> List[tuple]:
    n = C.c_size_t(0)
    _check(lib().cdp_get_trace(ctx, None, 0, C.byref(n)), ctx)
    buf = (cdp_trace_rec * max(1, n.value))()
    _check(lib().cdp_get_trace(ctx, buf, n.value, C.byref(n)), ctx)
    return [(r.tick, r.mb, r.step, r.stage, r.dir, r.version) for r in buf[:n.value]]


def cdp_get_live_counts(ctx) -> List[int]:
    n = C.c_size_t(0)
    _check(lib().cdp_get_live_counts(ctx, None, 0, C.byref(n)), ctx)
    buf = (C.c_int32 * max(1, n.value))()
    _check(lib().cdp_get_live_counts(ctx, buf, n.value, C.byref(n)), ctx)
    return list(buf[:n.value])


def cdp_get_live_bytes(ctx, kind: int = 0) -> List[int]:
    n = C.c_size_t(0)
    _check(lib().cdp_get_live_bytes(ctx, kind, None, 0, C.byref(n)), ctx)
    buf = (C.c_int64 * max(1, n.value))()
    _check(lib().cdp_get_live_bytes(ctx, kind, buf, n.value, C.byref(n)), ctx)
    return list(buf[:n.value])


def cdp_get_stats(ctx) -> dict:
    s = cdp_stats()
    _check(lib().cdp_get_stats(ctx, C.byref(s)), ctx)
    return {n: int(getattr(s, n)) for n, _ in cdp_stats._fields_}


def cdp_profile_gemm(ctx, enable: bool) -> None:
    _check(lib().cdp_profile_gemm(ctx, int(bool(enable))), ctx)


def cdp_get_gemm_profile(ctx) -> dict:
    p = cdp_gemm_profile()
    _check(lib().cdp_get_gemm_profile(ctx, C.byref(p)), ctx)
    return dict(launches=int(p.launches), total_ms=float(p.total_ms), flops=float(p.flops), bytes=float(p.bytes),
                empty_pair_ms=float(p.empty_pair_ms))


def cdp_destroy(ctx) -> None:
    lib().cdp_destroy(ctx)


def cdp_k_gemm(dtype, tile_shape, a_kmajor, b_kmajor, A_ptr, B_ptr, C_ptr, M, N, K, lda, ldb, stream=0) -> None:
    rc = lib().cdp_k_gemm(dtype, tile_shape, a_kmajor, b_kmajor, A_ptr, B_ptr, C_ptr, M, N, K, lda, ldb, stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_gemm")


def cdp_k_conv(dtype, which, in0_ptr, in1_ptr, out_ptr, B, H, W, Cin, Cout, ks, stride, pad, ws_ptr=0, ws_bytes=0,
               stream=0) -> None:
    rc = lib().cdp_k_conv(dtype, which, in0_ptr, in1_ptr, out_ptr, B, H, W, Cin, Cout, ks, stride, pad, ws_ptr or None,
                          ws_bytes, stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_conv")


def cdp_k_conv_wgrad_static(dtype, dy_ptr, x_ptr, dw_ptr, B, H, W, Cin, Cout, ks, stride, pad, stream=0) -> None:
    rc = lib().cdp_k_conv_wgrad_static(dtype, dy_ptr, x_ptr, dw_ptr, B, H, W, Cin, Cout, ks, stride, pad, stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_conv_wgrad_static: " + lib().cdp_last_error(None).decode())


def cdp_k_layernorm(dtype, backward, x_ptr, dy_ptr, add_ptr, gamma_ptr, beta_ptr, out_ptr, dgamma_ptr, dbeta_ptr, ws_ptr,
                    ws_bytes, rows, C_, stream=0) -> None:
    rc = lib().cdp_k_layernorm(dtype, backward, x_ptr, dy_ptr or None, add_ptr or None, gamma_ptr, beta_ptr or None, out_ptr,
                               dgamma_ptr or None, dbeta_ptr or None, ws_ptr or None, ws_bytes, rows, C_, stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_layernorm")


def cdp_k_gelu(dtype, backward, x_ptr, dy_ptr, out_ptr, n, stream=0) -> None:
    rc = lib().cdp_k_gelu(dtype, backward, x_ptr, dy_ptr or None, out_ptr, n, stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_gelu")


def cdp_k_attention(dtype, backward, qkv_ptr, P_ptr, dout_ptr, out_ptr, ws_ptr, ws_bytes, B, T, D, heads, stream=0) -> None:
    rc = lib().cdp_k_attention(dtype, backward, qkv_ptr, P_ptr, dout_ptr or None, out_ptr, ws_ptr, ws_bytes, B, T, D, heads,
                               stream or None)
    if rc != CDP_OK:
        raise CdpError(rc, "cdp_k_attention")


# ---- convenience wrapper used by tests and bench -------------------------------------------
class Trainer:
    """Owns a context plus (for GPU runs) the torch tensor that backs the arena."""

    def __init__(self, stages, in_shape, N: int, B: int, lr: float, rule: int, dtype: int, dry_run: bool = False,
                 device: str = "cuda:0", momentum: float = 0.0, weight_decay: float = 0.0, dp_batched: bool = False,
                 fresh_mask=None, bwd_fresh: bool = False, dw_group: int = 1):
        self.N, self.B, self.S = N, B, len(stages)
        self.ctx = None
        self._arena = None
        if fresh_mask is not None and np.asarray(fresh_mask).shape != (N, len(stages)):
            raise ValueError("fresh_mask must have shape (N, S)")
        opts = make_opts(dtype, in_shape, dry_run=dry_run, momentum=momentum, weight_decay=weight_decay,
                         dp_batched=dp_batched, fresh_mask=fresh_mask, bwd_fresh=bwd_fresh, dw_group=dw_group)
        if not dry_run:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("libcdp needs a GPU (use dry_run=True for host-only bookkeeping)")
            need = cdp_arena_bytes(stages, N, B, rule, opts)
            self._arena = torch.empty(need + 256, dtype=torch.uint8, device=device)
            base = (self._arena.data_ptr() + 255) // 256 * 256
            stream = torch.cuda.current_stream(self._arena.device).cuda_stream
            opts = make_opts(dtype, in_shape, stream=stream, arena=base, arena_bytes=need, momentum=momentum,
                             weight_decay=weight_decay, dp_batched=dp_batched, fresh_mask=fresh_mask,
                             bwd_fresh=bwd_fresh, dw_group=dw_group)
            self.arena_bytes = need
        self.ctx = cdp_init(stages, N, B, lr, rule, opts)

    def set_weights(self, params_per_stage) -> None:
        for j, plist in enumerate(params_per_stage):
            flat = np.concatenate([np.asarray(p, dtype=np.float32).ravel() for p in plist]) if len(plist) else np.zeros(0, np.float32)
            cdp_set_weights(self.ctx, j, flat)

    def step(self, x, y) -> None:
        """x: float32 [N*B, ...], y: int32 [N*B]; torch tensors on the arena's device."""
        cdp_step(self.ctx, x.data_ptr(), y.data_ptr())

    def tick(self, x=None, y=None) -> None:
        cdp_tick(self.ctx, x.data_ptr() if x is not None else 0, y.data_ptr() if y is not None else 0)

    def tick_dry(self, has_data: bool = True) -> None:
        cdp_tick(self.ctx, 256 if has_data else 0, 256 if has_data else 0)

    def drain(self) -> None:
        cdp_drain(self.ctx)

    def weights(self, stage: int, version: int = -1) -> np.ndarray:
        return cdp_get_weights(self.ctx, stage, version)

    def losses(self, step: int) -> np.ndarray:
        return cdp_get_losses(self.ctx, step, self.N)

    def trace(self):
        return cdp_get_trace(self.ctx)

    def live_counts(self):
        return cdp_get_live_counts(self.ctx)

    def live_bytes(self, kind: int = 0):
        return cdp_get_live_bytes(self.ctx, kind)

    def stats(self) -> dict:
        return cdp_get_stats(self.ctx)

    def profile_gemm(self, enable: bool) -> None:
        cdp_profile_gemm(self.ctx, enable)

    def gemm_profile(self) -> dict:
        return cdp_get_gemm_profile(self.ctx)

    def close(self) -> None:
        if self.ctx is not None:
            cdp_destroy(self.ctx)
            self.ctx = None
        self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
