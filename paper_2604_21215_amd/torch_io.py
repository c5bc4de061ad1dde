"""Host <-> device plumbing with PyTorch (device memory only; no arithmetic of the method)."""
from __future__ import annotations

import numpy as np
import torch

from . import binding
from . import inputs as gen


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """float32 host array -> device tensor in the storage dtype (bf16 values must already be bf16-exact)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        bits = gen.f32_to_bf16_bits(a).view(np.int16).reshape(a.shape)
        return torch.from_numpy(bits).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> float64 host array (exact widening)."""
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return gen.bf16_bits_to_f32(bits).reshape(bits.shape).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class DeviceLayer:
    """Weights of one layer resident on the device plus the marshalled rt_layer_weights struct."""

    def __init__(self, weights: dict, gains: dict | None, dtype: str, device="cuda:0", alias_kv_gain=False):
        self.t = {k: to_device(v, dtype, device) for k, v in weights.items()}
        if gains is not None:
            for k, v in gains.items():
                if k == "g_kv" and alias_kv_gain:
                    continue
                self.t[k] = to_device(v, dtype, device)
        self.struct = binding.make_weights(self.t)


def prefill(ctx: binding.RTContext, layer: DeviceLayer, x_dev: torch.Tensor, kv_cap: int | None = None):
    """Allocate outputs, call rt_layer_prefill, return device tensors (no synchronisation)."""
    B, N, d = x_dev.shape
    H = ctx.cfg.n_heads
    kv_cap = N if kv_cap is None else kv_cap
    y = torch.empty_like(x_dev)
    K = torch.zeros((kv_cap, B, H, d // H), dtype=x_dev.dtype, device=x_dev.device)
    V = torch.zeros_like(K)
    ctx.rt_layer_prefill(layer.struct, x_dev, y, K, V)
    return y, K, V
