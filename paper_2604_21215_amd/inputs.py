"""Seeded synthetic inputs for the Recurrent Transformer (RT) layer workloads.

This module holds no arithmetic of the method itself: it only draws numbers and
rounds them to the storage dtype.  Both the CPU oracle's tests and the GPU path
are fed from the arrays made here, so the two sides see identical buffers.

Generator: a counter-based hash (splitmix64 finaliser applied to
``key(seed, stream) + counter``) turned into standard normals with Box-Muller.
Element ``(b, n, k)`` of the activations has a counter that does not depend on
the batch size or the sequence length, so a shorter sequence is a prefix of a
longer one drawn with the same seed (used by the sequence-length sweep).

The workloads have no dataset behind them: the paper's latency protocol (Sec. 6,
"The setup") times one layer on shape-only inputs, and every configuration here
is x ~ N(0,1), weight matrices ~ N(0, 0.02^2), unit gains, no biases.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np

_U64 = np.uint64
_MASK = (1 << 64) - 1


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
    return z ^ (z >> _U64(31))


def _key(seed: int, stream: int) -> np.uint64:
    k = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _MASK
    with np.errstate(over="ignore"):
        return _mix64(np.array([k], dtype=_U64))[0]


def normal_from_counters(seed: int, stream: int, counters: np.ndarray) -> np.ndarray:
    """Standard normals (float64), one per counter, reproducible per (seed, stream)."""
    c = np.ascontiguousarray(counters, dtype=_U64)
    with np.errstate(over="ignore"):
        h = _mix64(_mix64(c + _key(seed, stream)) + _U64(0x9E3779B97F4A7C15))
    hi = (h >> _U64(32)).astype(np.float64)
    lo = (h & _U64(0xFFFFFFFF)).astype(np.float64)
    u1 = (hi + 0.5) / 4294967296.0
    u2 = (lo + 0.5) / 4294967296.0
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def uniform_ints_from_counters(seed: int, stream: int, counters: np.ndarray, high: int) -> np.ndarray:
    c = np.ascontiguousarray(counters, dtype=_U64)
    with np.errstate(over="ignore"):
        h = _mix64(_mix64(c + _key(seed, stream)) + _U64(0x9E3779B97F4A7C15))
    return ((h >> _U64(11)) % _U64(high)).astype(np.int64)


def normal(seed: int, stream: int, shape, scale: float = 1.0) -> np.ndarray:
    """float32 array of N(0, scale^2) values; element i (C order) uses counter i."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    step = 1 << 22
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = (normal_from_counters(seed, stream, np.arange(s, e, dtype=_U64)) * scale).astype(np.float32)
    return out.reshape(shape)


def activations(seed: int, stream: int, B: int, N: int, d: int) -> np.ndarray:
    """x[B, N, d] ~ N(0,1), float32.  Counter of (b, n, k) is b*2^40 + n*2^20 + k."""
    assert N < (1 << 20) and d < (1 << 20)
    out = np.empty((B, N, d), dtype=np.float32)
    k = np.arange(d, dtype=_U64)
    rows_per = max(1, (1 << 22) // d)
    for b in range(B):
        for s in range(0, N, rows_per):
            e = min(N, s + rows_per)
            n = np.arange(s, e, dtype=_U64)
            c = (_U64(b) << _U64(40)) + (n[:, None] << _U64(20)) + k[None, :]
            out[b, s:e, :] = normal_from_counters(seed, stream, c.ravel()).reshape(e - s, d).astype(np.float32)
    return out


# ----------------------------------------------------------------------------------------------
# bf16 storage rounding (round to nearest, ties to even) -- an encoding, not part of the method.
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(np.shape(a))


# ----------------------------------------------------------------------------------------------
# Workload table: the five benchmark configurations.
# ----------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16"  (storage dtype of x, y, K, V and weights)
    B: int
    N: int
    d: int
    H: int
    F: int
    layers: int = 1
    vocab: int = 0
    decode_steps: int = 0
    seed: int = 0
    head_dim: int = 64

    @property
    def resid_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.layers))


_SEED0 = 20260421 * 16

WORKLOADS = {
    "cfg1": Workload("cfg1", "f32", 1, 256, 128, 2, 512, seed=_SEED0 + 1),
    "cfg2": Workload("cfg2", "bf16", 8, 1024, 768, 12, 3072, seed=_SEED0 + 2),
    "cfg3": Workload("cfg3", "bf16", 8, 2048, 1024, 16, 4096, seed=_SEED0 + 3),
    "cfg4_1024": Workload("cfg4_1024", "bf16", 2, 1024, 1024, 16, 4096, seed=_SEED0 + 4),
    "cfg4_2048": Workload("cfg4_2048", "bf16", 2, 2048, 1024, 16, 4096, seed=_SEED0 + 4),
    "cfg4_4096": Workload("cfg4_4096", "bf16", 2, 4096, 1024, 16, 4096, seed=_SEED0 + 4),
    "cfg4_8192": Workload("cfg4_8192", "bf16", 2, 8192, 1024, 16, 4096, seed=_SEED0 + 4),
    "cfg5": Workload("cfg5", "bf16", 4, 4096, 1024, 16, 4096, layers=12, vocab=32768,
                     decode_steps=128, seed=_SEED0 + 5),
}

_WEIGHT_ORDER = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")


@dataclass
class LayerInputs:
    """Host buffers of one layer call.  All arrays are float32; for a bf16 workload
    every value is already rounded to bf16, so widening to float64 (oracle) and
    narrowing to bf16 (GPU) are both exact."""
    x: np.ndarray                                   # [B, N, d]
    weights: dict = field(default_factory=dict)    # Wq,Wk,Wv,Wo [d,d]; W1 [F,d]; W2 [d,F]; row-major [out,in]
    gains: dict = field(default_factory=dict)      # g_attn,g_mlp,g_kv [d]; g_q,g_k [d] (= [H, head_dim])


def weight_shapes(d: int, F: int) -> dict:
    return {"Wq": (d, d), "Wk": (d, d), "Wv": (d, d), "Wo": (d, d), "W1": (F, d), "W2": (d, F)}


def make_layer_weights(seed: int, layer: int, d: int, F: int, dtype: str, std: float = 0.02) -> dict:
    shapes = weight_shapes(d, F)
    w = {}
    for i, name in enumerate(_WEIGHT_ORDER):
        a = normal(seed, 100 + 16 * layer + i, shapes[name], std)
        w[name] = round_to_bf16(a) if dtype == "bf16" else a
    return w


def unit_gains(d: int) -> dict:
    one = np.ones(d, dtype=np.float32)
    return {k: one.copy() for k in ("g_attn", "g_mlp", "g_kv", "g_q", "g_k")}


def random_gains(seed: int, d: int, dtype: str, spread: float = 0.25) -> dict:
    """Non-trivial gains (1 + spread*N(0,1)) for tests that must exercise the gain paths."""
    g = {}
    for i, k in enumerate(("g_attn", "g_mlp", "g_kv", "g_q", "g_k")):
        a = (1.0 + spread * normal(seed, 900 + i, (d,))).astype(np.float32)
        g[k] = round_to_bf16(a) if dtype == "bf16" else a
    return g


def make_layer_inputs(wl: Workload, layer: int = 0, *, B: int | None = None, N: int | None = None) -> LayerInputs:
    """x and the weights of layer `layer` for a workload (optionally a smaller B / N prefix)."""
    B = wl.B if B is None else B
    N = wl.N if N is None else N
    x = activations(wl.seed, 1, B, N, wl.d)
    if wl.dtype == "bf16":
        x = round_to_bf16(x)
    return LayerInputs(x=x, weights=make_layer_weights(wl.seed, layer, wl.d, wl.F, wl.dtype), gains=unit_gains(wl.d))


def make_custom(seed: int, dtype: str, B: int, N: int, d: int, H: int, F: int, *, x_scale: float = 1.0,
                w_std: float = 0.02, gains: str = "unit") -> LayerInputs:
    """Free-form shapes for unit tests and edge cases (same generator, same draw order)."""
    x = activations(seed, 1, B, N, d) * np.float32(x_scale)
    if dtype == "bf16":
        x = round_to_bf16(x)
    g = unit_gains(d) if gains == "unit" else random_gains(seed, d, dtype)
    return LayerInputs(x=x, weights=make_layer_weights(seed, 0, d, F, dtype, w_std), gains=g)


def make_token_ids(wl: Workload) -> np.ndarray:
    """ids[B, N + decode_steps] uniform over the vocabulary (stack workload)."""
    T = wl.N + wl.decode_steps
    c = np.arange(wl.B * T, dtype=_U64)
    return uniform_ints_from_counters(wl.seed, 2, c, wl.vocab).reshape(wl.B, T)


def make_embedding_tables(wl: Workload) -> dict:
    emb = normal(wl.seed, 3, (wl.vocab, wl.d), 0.02)
    head = normal(wl.seed, 4, (wl.vocab, wl.d), 0.02)
    if wl.dtype == "bf16":
        emb, head = round_to_bf16(emb), round_to_bf16(head)
    return {"embedding": emb, "lm_head": head, "g_final": np.ones(wl.d, dtype=np.float32)}
