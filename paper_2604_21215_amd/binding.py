"""ctypes binding of librt_hip.so: the same entry points as include/rt.h, argument marshalling only.

Every step of the layer runs in the library's HIP kernels; PyTorch is used by callers for device
memory and streams.  There is no CPU fallback: if the library is missing the import of the symbols
fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
import sys as _sys

from . import build as _build

RT_OK = 0
RT_ERR_INVALID_ARG, RT_ERR_UNSUPPORTED, RT_ERR_OOM, RT_ERR_HIP, RT_ERR_STATE = 1, 2, 3, 4, 5
RT_F32, RT_BF16 = 0, 1
RT_FLAG_NORM_FREE = 0x1
RT_FLAG_ENGINE_STEPWISE = 0x2
RT_FLAG_ENGINE_PERSISTENT = 0x4
RT_FLAG_NO_MFMA = 0x8
RT_FLAG_HIP_GRAPH = 0x10
RT_FLAG_DEBUG_POISON = 0x20
RT_RESERVE_LOOP_FREE, RT_RESERVE_BACKWARD = 0x1, 0x2

EXPORTS = ("rt_create", "rt_layer_prefill", "rt_decode_step", "rt_destroy", "rt_last_error", "rt_status_string",
           "rt_workspace_bytes", "rt_device_wait_expired", "rt_engine_name", "rt_schedule_events", "rt_partial_slot",
           "rt_version", "rt_phase_trace", "rt_schedule_events_shifted", "rt_embed_rows", "rt_lm_head", "rt_cross_block_event",
           "rt_stack_prefill", "rt_schedule_events_chunked", "rt_layer_recompute", "rt_transformer_layer",
           "rt_layer_prefill_blocked", "rt_decode_step_static", "rt_layer_backward", "rt_decode_phase_trace")


class rt_config(C.Structure):
    _fields_ = [
        ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("d_hidden", C.c_int32),
        ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("dtype", C.c_int32), ("p_min", C.c_int32),
        ("resid_scale", C.c_float), ("attn_scale", C.c_float), ("rms_eps", C.c_float), ("flags", C.c_uint32),
        ("device", C.c_int32), ("stream", C.c_void_p), ("alibi_max_bias", C.c_float),
        ("reserve_stack_layers", C.c_int32), ("reserve_stack_chunk", C.c_int32), ("reserve", C.c_uint32),
    ]


class rt_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2", "g_attn", "g_mlp", "g_kv", "g_q", "g_k")]


class rt_layer_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Wq", "Wk", "Wv", "Wo", "W1", "W2", "g_attn", "g_mlp", "g_kv", "g_q", "g_k")]


class RTError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (status, msg))
        self.status = status


_lib = None


def load():
    """Load the built library (builds it only if no library is there at all)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_hip(True)
    try:
        # callers hold their device memory in torch tensors: load torch's HIP runtime first so that the library binds
        # to the same one whatever the import order (two runtimes in one process do not share a device context)
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(_build.LIB)
    ctxp = C.c_void_p
    L.rt_create.argtypes = [C.POINTER(rt_config), C.POINTER(ctxp)]
    L.rt_create.restype = C.c_int
    L.rt_layer_prefill.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_layer_prefill.restype = C.c_int
    L.rt_decode_step.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                 C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_decode_step.restype = C.c_int
    L.rt_destroy.argtypes = [ctxp]
    L.rt_destroy.restype = C.c_int
    L.rt_last_error.argtypes = [ctxp]
    L.rt_last_error.restype = C.c_char_p
    L.rt_status_string.argtypes = [C.c_int]
    L.rt_status_string.restype = C.c_char_p
    L.rt_workspace_bytes.argtypes = [ctxp]
    L.rt_workspace_bytes.restype = C.c_uint64
    L.rt_device_wait_expired.argtypes = [ctxp]
    L.rt_device_wait_expired.restype = C.c_int32
    L.rt_engine_name.argtypes = [ctxp]
    L.rt_engine_name.restype = C.c_char_p
    L.rt_schedule_events.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32]
    L.rt_schedule_events.restype = C.c_int32
    L.rt_schedule_events_shifted.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32]
    L.rt_schedule_events_shifted.restype = C.c_int32
    L.rt_schedule_events_chunked.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32]
    L.rt_schedule_events_chunked.restype = C.c_int32
    L.rt_partial_slot.argtypes = [C.c_int32, C.c_int32]
    L.rt_partial_slot.restype = C.c_int64
    L.rt_version.restype = C.c_int32
    L.rt_phase_trace.argtypes = [ctxp, C.POINTER(C.c_uint64), C.c_int32]
    L.rt_phase_trace.restype = C.c_int32
    L.rt_decode_phase_trace.argtypes = [ctxp, C.POINTER(C.c_uint64), C.c_int32]
    L.rt_decode_phase_trace.restype = C.c_int32
    L.rt_embed_rows.argtypes = [ctxp, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                C.c_void_p]
    L.rt_embed_rows.restype = C.c_int
    L.rt_lm_head.argtypes = [ctxp, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    L.rt_lm_head.restype = C.c_int
    L.rt_cross_block_event.argtypes = [ctxp, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    L.rt_cross_block_event.restype = C.c_int
    L.rt_stack_prefill.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                   C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32, C.c_int32]
    L.rt_stack_prefill.restype = C.c_int
    L.rt_layer_recompute.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_layer_recompute.restype = C.c_int
    L.rt_transformer_layer.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_transformer_layer.restype = C.c_int
    L.rt_layer_prefill_blocked.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_layer_prefill_blocked.restype = C.c_int
    L.rt_decode_step_static.argtypes = [C.POINTER(rt_config), C.POINTER(rt_layer_weights), C.c_void_p, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32]
    L.rt_decode_step_static.restype = C.c_int
    L.rt_layer_backward.argtypes = [ctxp, C.POINTER(rt_layer_weights), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(rt_layer_grads)]
    L.rt_layer_backward.restype = C.c_int
    _lib = L
    return L


def _check(L, ctx, rc):
    if rc != RT_OK:
        msg = L.rt_last_error(ctx).decode() if ctx else ""
        raise RTError(L.rt_status_string(rc).decode(), msg)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def rt_decode_step_static(cfg: rt_config, weights: rt_layer_weights, x_t, t, y_t, K, V):
    """rt_decode_step_static(cfg, w, x_t[B,d], B, t, y_t, K, V, kv_cap): the decoding step without a context."""
    L = load()
    rc = L.rt_decode_step_static(C.byref(cfg), C.byref(weights), _ptr(x_t), x_t.shape[0], int(t), _ptr(y_t), _ptr(K), _ptr(V),
                                 K.shape[0])
    if rc != RT_OK:
        raise RTError(L.rt_status_string(rc).decode(), L.rt_last_error(None).decode())


def raw_decode_static(cfg, weights, x_ptr, B, t, y_ptr, K_ptr, V_ptr, kv_cap) -> int:
    """Status code of rt_decode_step_static on raw addresses (error-path tests)."""
    return load().rt_decode_step_static(C.byref(cfg), C.byref(weights), C.c_void_p(x_ptr), B, t, C.c_void_p(y_ptr),
                                        C.c_void_p(K_ptr), C.c_void_p(V_ptr), kv_cap)


def make_weights(w: dict) -> rt_layer_weights:
    """w maps names to device tensors (or None for the optional gains)."""
    s = rt_layer_weights()
    for name, _ in rt_layer_weights._fields_:
        t = w.get(name)
        setattr(s, name, None if t is None else t.data_ptr())
    return s


def _events(fn, N, p_min):
    n = fn(N, p_min, None, 0)
    if n < 0:
        raise RTError("RT_ERR_INVALID_ARG", "schedule")
    buf = (C.c_int32 * (5 * max(n, 1)))()
    fn(N, p_min, buf, n)
    return [tuple(buf[5 * i + j] for j in range(5)) for i in range(n)]


def rt_schedule_events(N: int, p_min: int):
    return _events(load().rt_schedule_events, N, p_min)


def rt_schedule_events_shifted(N: int, p_min: int):
    return _events(load().rt_schedule_events_shifted, N, p_min)


def rt_schedule_events_chunked(N: int, p_min: int, chunk: int):
    fn = load().rt_schedule_events_chunked
    return _events(lambda n, p, buf, cap: fn(n, p, chunk, buf, cap), N, p_min)


def rt_partial_slot(level: int, query: int) -> int:
    return int(load().rt_partial_slot(level, query))


class RTContext:
    """Owns an rt_ctx.  Methods mirror the C entry points and take torch device tensors."""

    def __init__(self, d_model, n_heads, d_hidden, max_batch, max_seq, dtype, *, p_min=0, resid_scale=1.0,
                 attn_scale=1.0, rms_eps=1e-6, flags=0, device=0, stream=None, alibi_max_bias=0.0, reserve_stack_layers=0,
                 reserve_stack_chunk=0, reserve=0):
        L = load()
        cfg = rt_config(d_model, n_heads, d_model // n_heads if n_heads else 0, d_hidden, max_batch, max_seq,
                        RT_BF16 if dtype in ("bf16", RT_BF16) and dtype != 0 else RT_F32, p_min, resid_scale, attn_scale,
                        rms_eps, flags, device, stream, alibi_max_bias, reserve_stack_layers, reserve_stack_chunk, reserve)
        self.cfg = cfg
        self._L = L
        self._ctx = C.c_void_p()
        rc = L.rt_create(C.byref(cfg), C.byref(self._ctx))
        if rc != RT_OK:
            raise RTError(L.rt_status_string(rc).decode(), "rt_create")

    # -- rt_layer_prefill(ctx, w, x[B,N,d], B, N, y, K, V, kv_cap)
    def rt_layer_prefill(self, weights: rt_layer_weights, x, y, K, V):
        B, N, _ = x.shape
        rc = self._L.rt_layer_prefill(self._ctx, C.byref(weights), _ptr(x), B, N, _ptr(y), _ptr(K), _ptr(V), K.shape[0])
        _check(self._L, self._ctx, rc)

    # -- rt_stack_prefill(ctx, layers[L], L, x[B,N,d], B, N, y[L], K[L], V[L], kv_cap, chunk)
    def rt_stack_prefill(self, weights: list, x, ys: list, Ks: list, Vs: list, chunk: int = 0):
        B, N, _ = x.shape
        L = len(weights)
        warr = (rt_layer_weights * L)(*weights)
        parr = lambda ts: (C.c_void_p * L)(*[t.data_ptr() for t in ts])
        rc = self._L.rt_stack_prefill(self._ctx, warr, L, _ptr(x), B, N, parr(ys), parr(Ks), parr(Vs), Ks[0].shape[0],
                                      int(chunk))
        _check(self._L, self._ctx, rc)

    def raw_stack_prefill(self, weights: list, x_ptr, B, N, y_ptrs, K_ptrs, V_ptrs, kv_cap, chunk) -> int:
        """Status code of rt_stack_prefill on raw addresses (error-path tests)."""
        L = len(weights)
        warr = (rt_layer_weights * L)(*weights)
        parr = lambda ps: (C.c_void_p * L)(*ps)
        return self._L.rt_stack_prefill(self._ctx, warr, L, C.c_void_p(x_ptr), B, N, parr(y_ptrs), parr(K_ptrs),
                                        parr(V_ptrs), kv_cap, chunk)

    # -- rt_layer_recompute(ctx, w, x[B,N,d], z[B,N,d], B, N, y, K, V, kv_cap)
    def rt_layer_recompute(self, weights: rt_layer_weights, x, z, y, K, V):
        B, N, _ = x.shape
        rc = self._L.rt_layer_recompute(self._ctx, C.byref(weights), _ptr(x), _ptr(z), B, N, _ptr(y), _ptr(K), _ptr(V),
                                        K.shape[0])
        _check(self._L, self._ctx, rc)

    # -- rt_layer_backward(ctx, w, x[B,N,d], z[B,N,d], gy[B,N,d], gK | None, gV | None, B, N, dx[B,N,d] f32, grads)
    def rt_layer_backward(self, weights: rt_layer_weights, x, z, gy, gK, gV, dx, grads: dict):
        """grads: name -> fp32 device tensor (any subset of the six matrices and five gains)."""
        B, N, _ = x.shape
        g = rt_layer_grads()
        for name, _t in rt_layer_grads._fields_:
            t = grads.get(name)
            setattr(g, name, None if t is None else t.data_ptr())
        rc = self._L.rt_layer_backward(self._ctx, C.byref(weights), _ptr(x), _ptr(z), _ptr(gy), _ptr(gK), _ptr(gV), B, N,
                                       _ptr(dx), C.byref(g))
        _check(self._L, self._ctx, rc)

    # -- rt_layer_prefill_blocked(ctx, w, x[B,N,d], B, N, block, y, K, V, kv_cap)
    def rt_layer_prefill_blocked(self, weights: rt_layer_weights, x, block, y, K, V):
        B, N, _ = x.shape
        rc = self._L.rt_layer_prefill_blocked(self._ctx, C.byref(weights), _ptr(x), B, N, int(block), _ptr(y), _ptr(K),
                                              _ptr(V), K.shape[0])
        _check(self._L, self._ctx, rc)

    # -- rt_transformer_layer(ctx, w, x[B,N,d], B, N, y, K, V, kv_cap)
    def rt_transformer_layer(self, weights: rt_layer_weights, x, y, K, V):
        B, N, _ = x.shape
        rc = self._L.rt_transformer_layer(self._ctx, C.byref(weights), _ptr(x), B, N, _ptr(y), _ptr(K), _ptr(V), K.shape[0])
        _check(self._L, self._ctx, rc)

    # -- rt_decode_step(ctx, w, x_t[B,d], B, t, y_t, K, V, kv_cap)
    def rt_decode_step(self, weights: rt_layer_weights, x_t, t, y_t, K, V):
        rc = self._L.rt_decode_step(self._ctx, C.byref(weights), _ptr(x_t), x_t.shape[0], int(t), _ptr(y_t), _ptr(K),
                                    _ptr(V), K.shape[0])
        _check(self._L, self._ctx, rc)

    # -- rt_embed_rows(ctx, table[vocab,d], vocab, ids[B,ids_stride] int32, ids_stride, first, B, N, x[B,N,d])
    def rt_embed_rows(self, table, ids, first, x):
        B, N, _ = x.shape
        rc = self._L.rt_embed_rows(self._ctx, _ptr(table), table.shape[0], _ptr(ids), ids.stride(0), int(first), B, N,
                                   _ptr(x))
        _check(self._L, self._ctx, rc)

    # -- rt_lm_head(ctx, W_lm[vocab,d], g_final[d] | None, vocab, z rows (stride z_stride elements), z_stride, B, logits[B,vocab] f32)
    def rt_lm_head(self, W_lm, g_final, z, z_stride, B, logits):
        rc = self._L.rt_lm_head(self._ctx, _ptr(W_lm), _ptr(g_final), W_lm.shape[0], _ptr(z), int(z_stride), int(B),
                                _ptr(logits))
        _check(self._L, self._ctx, rc)

    # -- rt_cross_block_event(ctx, K, V, B, t1, P, nq)
    def rt_cross_block_event(self, K, V, t1, P, nq):
        rc = self._L.rt_cross_block_event(self._ctx, _ptr(K), _ptr(V), K.shape[1], int(t1), int(P), int(nq))
        _check(self._L, self._ctx, rc)

    def raw_embed(self, table_ptr, vocab, ids_ptr, ids_stride, first, B, N, x_ptr) -> int:
        return self._L.rt_embed_rows(self._ctx, C.c_void_p(table_ptr), vocab, C.c_void_p(ids_ptr), ids_stride, first, B, N,
                                     C.c_void_p(x_ptr))

    def raw_lm_head(self, W_ptr, g_ptr, vocab, z_ptr, z_stride, B, logits_ptr) -> int:
        return self._L.rt_lm_head(self._ctx, C.c_void_p(W_ptr), C.c_void_p(g_ptr), vocab, C.c_void_p(z_ptr), z_stride, B,
                                  C.c_void_p(logits_ptr))

    def raw_prefill(self, weights, x_ptr, B, N, y_ptr, K_ptr, V_ptr, kv_cap) -> int:
        """Status code of rt_layer_prefill on raw addresses (error-path tests)."""
        return self._L.rt_layer_prefill(self._ctx, C.byref(weights) if weights is not None else None, C.c_void_p(x_ptr),
                                        B, N, C.c_void_p(y_ptr), C.c_void_p(K_ptr), C.c_void_p(V_ptr), kv_cap)

    def raw_decode(self, weights, x_ptr, B, t, y_ptr, K_ptr, V_ptr, kv_cap) -> int:
        return self._L.rt_decode_step(self._ctx, C.byref(weights) if weights is not None else None, C.c_void_p(x_ptr),
                                      B, t, C.c_void_p(y_ptr), C.c_void_p(K_ptr), C.c_void_p(V_ptr), kv_cap)

    def last_error(self) -> str:
        return self._L.rt_last_error(self._ctx).decode()

    def engine_name(self) -> str:
        return self._L.rt_engine_name(self._ctx).decode()

    def workspace_bytes(self) -> int:
        return int(self._L.rt_workspace_bytes(self._ctx))

    def device_wait_expired(self) -> int:
        return int(self._L.rt_device_wait_expired(self._ctx))

    def phase_trace(self, rows: int):
        """[rows, 16] clock stamps (100 MHz) of the persistent engine, or None when tracing is off."""
        import numpy as np
        buf = np.zeros((rows, 16), dtype=np.uint64)
        n = self._L.rt_phase_trace(self._ctx, buf.ctypes.data_as(C.POINTER(C.c_uint64)), rows)
        return buf[:n] if n > 0 else None

    def decode_phase_trace(self, workgroups: int = 256):
        """[workgroups, 16] clock stamps (100 MHz) of the last single-launch decoding step, or None when tracing is off."""
        import numpy as np
        buf = np.zeros((workgroups, 16), dtype=np.uint64)
        n = self._L.rt_decode_phase_trace(self._ctx, buf.ctypes.data_as(C.POINTER(C.c_uint64)), workgroups)
        return buf[:n] if n > 0 else None

    def rt_destroy(self):
        if self._ctx:
            self._L.rt_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        if _sys is None or _sys.is_finalizing():   # no HIP calls while the interpreter (and the runtimes behind it) shut down
            return
        try:
            self.rt_destroy()
        except Exception:
            pass
