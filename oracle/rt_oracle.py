"""ctypes front end of the fp64 CPU oracle (oracle/rt_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module.
It builds the C file with gcc on first use (a second or two) and never touches the GPU
library.  All arrays are float64 numpy, C-contiguous:
    x, y : [B, N, d]        K, V : [kv_cap, B, H, dh]        weights : [out, in]
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rt_oracle.c")
_LIB = os.path.join(_HERE, "librt_oracle.so")

_MLP_FN = C.CFUNCTYPE(None, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int, C.c_void_p)
_DP = C.POINTER(C.c_double)


class _Params(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("H", C.c_int32), ("dh", C.c_int32), ("F", C.c_int32),
        ("alpha", C.c_double), ("attn_scale", C.c_double), ("eps", C.c_double),
        ("norm_free", C.c_int32), ("threads", C.c_int32),
        ("Wq", _DP), ("Wk", _DP), ("Wv", _DP), ("Wo", _DP), ("W1", _DP), ("W2", _DP),
        ("g_attn", _DP), ("g_mlp", _DP), ("g_kv", _DP), ("g_q", _DP), ("g_k", _DP),
        ("mlp", _MLP_FN), ("mlp_user", C.c_void_p),
        ("alibi_max_bias", C.c_double),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O3, no fast-math) into oracle/librt_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-fno-fast-math",
               "-ffp-contract=off", _SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (gcc, -O1, frame pointers kept) into `out`;
    a process that loads it needs gcc's libasan preloaded (tests/test_oracle_sanitized.py does that in a child)."""
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-fno-fast-math", "-ffp-contract=off", _SRC, "-o", out, "-lm"]
    subprocess.run(cmd, check=True)
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("RT_ORACLE_LIB")   # an already built variant of the same source (the sanitizer build)
        if not path:
            path = build()
        L = C.CDLL(path)
        PP = C.POINTER(_Params)
        L.rto_layer_prefill.argtypes = [PP, _DP, C.c_int, C.c_int, _DP, _DP, _DP, C.c_int, _DP]
        L.rto_layer_prefill.restype = C.c_int
        L.rto_layer_prefill_tiled.argtypes = [PP, _DP, C.c_int, C.c_int, _DP, _DP, _DP, C.c_int, C.c_int]
        L.rto_layer_prefill_tiled.restype = C.c_int
        L.rto_transformer_layer.argtypes = [PP, _DP, C.c_int, C.c_int, _DP, _DP, _DP, C.c_int, _DP]
        L.rto_transformer_layer.restype = C.c_int
        L.rto_decode_step.argtypes = [PP, _DP, C.c_int, C.c_int, _DP, _DP, _DP, C.c_int]
        L.rto_decode_step.restype = C.c_int
        L.rto_layer_prefill_blocked.argtypes = [PP, _DP, C.c_int, C.c_int, C.c_int, _DP, _DP, _DP, C.c_int]
        L.rto_layer_prefill_blocked.restype = C.c_int
        L.rto_update_tile.argtypes = [_DP, C.c_int, C.c_int, _DP, _DP, C.c_int, C.c_int, C.c_int, C.c_double,
                                      _DP, _DP, _DP, C.c_double, C.c_int]
        L.rto_update_tile.restype = None
        L.rto_schedule.argtypes = [C.c_int, C.POINTER(C.c_int32), C.c_int]
        L.rto_schedule.restype = C.c_int
        L.rto_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(_DP) if a is not None else _DP()


class Layer:
    """Parameters of one RT layer for the oracle.

    weights: dict with Wq, Wk, Wv [d,d], optional Wo [d,d] (missing/None = identity),
             W1 [F,d], W2 [d,F] (not needed when `mlp` is given).
    gains:   optional dict g_attn, g_mlp, g_kv, g_q, g_k (missing = ones; g_kv missing = g_attn).
    mlp:     optional Python callable  u(np.ndarray[d]) -> np.ndarray[d]  replacing the MLP block.
    """

    def __init__(self, weights, H, *, gains=None, alpha=1.0, attn_scale=1.0, eps=1e-6, norm_free=False,
                 mlp=None, threads=0, alibi_max_bias=0.0):
        self._keep = []
        w = {k: (_f64(v) if v is not None else None) for k, v in weights.items()}
        d = w["Wq"].shape[0]
        assert d % H == 0
        self.d, self.H, self.dh = d, H, d // H
        self.F = w["W1"].shape[0] if w.get("W1") is not None else 0
        g = dict(gains or {})
        if g.get("g_kv") is None and g.get("g_attn") is not None:
            g["g_kv"] = g["g_attn"]
        g = {k: (_f64(v) if v is not None else None) for k, v in g.items()}
        p = _Params()
        p.d, p.H, p.dh, p.F = d, H, self.dh, self.F
        p.alpha, p.attn_scale, p.eps = float(alpha), float(attn_scale), float(eps)
        p.norm_free, p.threads = int(bool(norm_free)), int(threads)
        p.alibi_max_bias = float(alibi_max_bias)
        self._w, self._g, self._mlp = w, g, mlp
        for name in ("Wq", "Wk", "Wv", "Wo", "W1", "W2"):
            a = w.get(name)
            setattr(p, name, _ptr(a))
            self._keep.append(a)
        for name in ("g_attn", "g_mlp", "g_kv", "g_q", "g_k"):
            a = g.get(name)
            setattr(p, name, _ptr(a))
            self._keep.append(a)
        if mlp is not None:
            def _cb(inp, out, n, _user, _f=mlp):
                u = np.ctypeslib.as_array(inp, shape=(n,)).copy()
                r = np.asarray(_f(u), dtype=np.float64)
                np.ctypeslib.as_array(out, shape=(n,))[:] = r
            self._cb = _MLP_FN(_cb)
            p.mlp = self._cb
        self.p = p

    # ------------------------------------------------------------------ entry points
    def _alloc(self, x, kv_cap):
        x = _f64(x)
        B, N, d = x.shape
        assert d == self.d
        kv_cap = N if kv_cap is None else kv_cap
        y = np.zeros((B, N, d))
        K = np.zeros((kv_cap, B, self.H, self.dh))
        V = np.zeros((kv_cap, B, self.H, self.dh))
        return x, B, N, kv_cap, y, K, V

    def prefill(self, x, kv_cap=None, want_attw=False):
        """Token-by-token recurrence of the RT layer definition.  Returns (y, K, V[, attw])."""
        x, B, N, kv_cap, y, K, V = self._alloc(x, kv_cap)
        aw = np.zeros((B, self.H, N, N)) if want_attw else None
        rc = lib().rto_layer_prefill(C.byref(self.p), _ptr(x), B, N, _ptr(y), _ptr(K), _ptr(V), kv_cap, _ptr(aw))
        if rc:
            raise RuntimeError("rto_layer_prefill failed: %d" % rc)
        return (y, K, V, aw) if want_attw else (y, K, V)

    def prefill_tiled(self, x, kv_cap=None, chunk=0):
        """Appendix C, Algorithms 1 + 2 literally (running statistics, tiled schedule).  chunk > 0: the variant
        in which a layer knows its queries one chunk ahead only (blocks of `chunk` keys and more replaced by one
        UpdateTile per chunk over all earlier keys)."""
        x, B, N, kv_cap, y, K, V = self._alloc(x, kv_cap)
        rc = lib().rto_layer_prefill_tiled(C.byref(self.p), _ptr(x), B, N, _ptr(y), _ptr(K), _ptr(V), kv_cap, int(chunk))
        if rc:
            raise RuntimeError("rto_layer_prefill_tiled failed: %d" % rc)
        return y, K, V

    def prefill_blocked(self, x, S, kv_cap=None):
        """Blocked recurrence (Sec. 8, one sentence; reading: persistent pairs across blocks of S positions, temporary
        pairs inside a block).  S = 1: the RT layer; S >= N: the Transformer layer.  Returns (y, K, V)."""
        x, B, N, kv_cap, y, K, V = self._alloc(x, kv_cap)
        rc = lib().rto_layer_prefill_blocked(C.byref(self.p), _ptr(x), B, N, int(S), _ptr(y), _ptr(K), _ptr(V), kv_cap)
        if rc:
            raise RuntimeError("rto_layer_prefill_blocked failed: %d" % rc)
        return y, K, V

    def recompute(self, x, z):
        """Sec. 6.1 ("Activation checkpointing"): the layer evaluated with its output z given.  All persistent pairs are
        projected from RMS(z) at once; position i then attends the persistent pairs of positions < i and its own
        temporary pair, and the output projection, residuals and MLP follow row by row - no sequential loop.  Dense
        numpy algebra, one (N x N) logit matrix per head.  Returns (y, K, V) in the layouts of prefill(); y equals z
        when z is the layer's output for x."""
        x, z = _f64(x), _f64(z)
        B, N, d = x.shape
        H, dh, p, w, g = self.H, self.dh, self.p, self._w, self._g
        eps, nf = p.eps, bool(p.norm_free)

        def rms(v, gain):
            if nf:
                return v
            r = v / np.sqrt(np.mean(v * v, axis=-1, keepdims=True) + eps)
            return r if gain is None else r * gain

        def heads(v, gain):      # per-head normalisation of [.., d] rows
            vh = v.reshape(v.shape[:-1] + (H, dh))
            return rms(vh, None if gain is None else gain.reshape(H, dh))

        n = rms(x, g.get("g_attn"))
        q = heads(n @ w["Wq"].T, g.get("g_q"))
        kt = heads(n @ w["Wk"].T, g.get("g_k"))
        vt = (n @ w["Wv"].T).reshape(B, N, H, dh)
        r = rms(z, g.get("g_kv"))
        Kp = heads(r @ w["Wk"].T, g.get("g_k"))
        Vp = (r @ w["Wv"].T).reshape(B, N, H, dh)
        dist = np.arange(N)[:, None] - np.arange(N)[None, :]          # i - j
        cat = np.zeros((B, N, H, dh))
        for b in range(B):
            for h in range(H):
                S = p.attn_scale * (q[b, :, h] @ Kp[b, :, h].T)
                if p.alibi_max_bias > 0:
                    S = S - 2.0 ** (-p.alibi_max_bias * (h + 1) / H) * dist
                S = np.where(dist > 0, S, -np.inf)                     # persistent pairs of earlier positions only
                own = p.attn_scale * np.sum(q[b, :, h] * kt[b, :, h], axis=-1)
                m = np.maximum(S.max(axis=1), own)
                E, e_own = np.exp(S - m[:, None]), np.exp(own - m)
                den = E.sum(axis=1) + e_own
                cat[b, :, h] = (E @ Vp[b, :, h] + e_own[:, None] * vt[b, :, h]) / den[:, None]
        a = cat.reshape(B, N, d)
        if w.get("Wo") is not None:
            a = a @ w["Wo"].T
        hdd = x + p.alpha * a
        u = rms(hdd, g.get("g_mlp"))
        if self._mlp is not None:
            mo = np.stack([[np.asarray(self._mlp(u[b, i]), dtype=np.float64) for i in range(N)] for b in range(B)])
        else:
            t = u @ w["W1"].T
            from math import sqrt
            from scipy.special import erf
            mo = (0.5 * t * (1.0 + erf(t / sqrt(2.0)))) @ w["W2"].T
        y = hdd + p.alpha * mo
        return y, np.ascontiguousarray(Kp.transpose(1, 0, 2, 3)), np.ascontiguousarray(Vp.transpose(1, 0, 2, 3))

    def transformer(self, x, want_attw=False):
        """Standard causal Transformer layer with the same parameters (Sec. 2.1)."""
        x, B, N, kv_cap, y, K, V = self._alloc(x, None)
        aw = np.zeros((B, self.H, N, N)) if want_attw else None
        rc = lib().rto_transformer_layer(C.byref(self.p), _ptr(x), B, N, _ptr(y), _ptr(K), _ptr(V), kv_cap, _ptr(aw))
        if rc:
            raise RuntimeError("rto_transformer_layer failed: %d" % rc)
        return (y, K, V, aw) if want_attw else (y, K, V)

    def decode_step(self, x_t, t, K, V):
        """One position given persistent rows 0..t-1 of K, V (modified in place at row t)."""
        x_t = _f64(x_t)
        B = x_t.shape[0]
        assert K.dtype == np.float64 and K.flags.c_contiguous and V.flags.c_contiguous
        y_t = np.zeros((B, self.d))
        rc = lib().rto_decode_step(C.byref(self.p), _ptr(x_t), B, int(t), _ptr(y_t), _ptr(K), _ptr(V), K.shape[0])
        if rc:
            raise RuntimeError("rto_decode_step failed: %d" % rc)
        return y_t


def update_tile(q, k, v, m, l, o, scale=1.0, slope=0.0, dist0=0):
    """Algorithm 2 on dense [nq,dh] / [nkv,dh] tiles; m, l [nq], o [nq,dh] updated in place.  slope, dist0: linear
    positional bias, query i being dist0 + i - j positions after key j."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    nq, dh = q.shape
    nkv = k.shape[0]
    for a in (m, l, o):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    lib().rto_update_tile(_ptr(q), nq, dh, _ptr(k), _ptr(v), nkv, dh, dh, float(scale), _ptr(m), _ptr(l), _ptr(o),
                          float(slope), int(dist0))


def schedule(N):
    """Events (t, P, u, v, s, e) of Algorithm 1, 1-based inclusive ranges."""
    cap = max(1, N)
    buf = (C.c_int32 * (6 * cap))()
    n = lib().rto_schedule(int(N), buf, cap)
    a = np.frombuffer(buf, dtype=np.int32).reshape(cap, 6)[:n].copy()
    return [tuple(int(v) for v in r) for r in a]


def max_threads():
    return int(lib().rto_max_threads())


def stack_prefill(layers, x0):
    """L stacked RT layers: the output of one layer is the input of the next (Sec. 2.2)."""
    out = []
    x = x0
    for lay in layers:
        y, K, V = lay.prefill(x)
        out.append((y, K, V))
        x = y
    return out


# ------------------------------------------------------------------ a stack of layers with embedding and read-out
def embed(table, ids):
    """First-layer input: row ids[b, n] of the embedding table (Sec. 2: token embeddings enter layer 1)."""
    return _f64(np.asarray(table)[np.asarray(ids)])


def lm_head(W_lm, z, g_final=None, eps=1e-6, norm_free=False):
    """logits = W_lm RMS(z; g_final) for rows z [B, d] (RMS as in Sec. 2, Notation; untied projection)."""
    z = _f64(z)
    if not norm_free:
        z = z / np.sqrt(np.mean(z * z, axis=-1, keepdims=True) + eps)
        if g_final is not None:
            z = z * _f64(g_final)
    return z @ _f64(W_lm).T


class Stack:
    """L RT layers (each its own parameters and key-value memory), embedding in front, read-out behind."""

    def __init__(self, layers, embedding, W_lm, g_final=None, eps=1e-6, norm_free=False):
        self.layers, self.embedding, self.W_lm, self.g_final = layers, embedding, W_lm, g_final
        self.eps, self.norm_free = eps, norm_free
        self.K, self.V = [], []

    def prefill(self, ids, N, kv_cap, progress=None):
        """Positions 0..N-1 of ids [B, >= N].  Returns (per-layer list of (y, K, V), logits of position N-1).
        progress: optional callable(layer index), called after each layer (long runs report through it)."""
        x = embed(self.embedding, np.asarray(ids)[:, :N])
        out = []
        self.K, self.V = [], []
        for l, lay in enumerate(self.layers):
            y, K, V = lay.prefill(x, kv_cap=kv_cap)
            if progress is not None:
                progress(l)
            out.append((y, K, V))
            self.K.append(K); self.V.append(V)
            x = y
        return out, lm_head(self.W_lm, x[:, N - 1], self.g_final, self.eps, self.norm_free)

    def decode_step(self, ids, t):
        """Position t over the caches held from prefill / earlier steps.  Returns (per-layer outputs [L, B, d], logits)."""
        x = embed(self.embedding, np.asarray(ids)[:, t])
        ys = []
        for l, lay in enumerate(self.layers):
            x = lay.decode_step(x, t, self.K[l], self.V[l])
            ys.append(x)
        return np.stack(ys), lm_head(self.W_lm, x, self.g_final, self.eps, self.norm_free)
