"""A stack of RT layers on the device: embedding -> L x rt_layer_prefill -> final norm + output projection,
and the same per decoding step over the per-layer caches (Sec. 2: the layers of one model are stacked,
each with its own key-value memory; Sec. 7.3: decoding).  Sequencing and pointer marshalling only: every
arithmetic step is a call into the C library."""
from __future__ import annotations

import torch

from . import binding
from .torch_io import DeviceLayer, to_device, torch_dtype


class DeviceStack:
    def __init__(self, ctx: binding.RTContext, layers: list[DeviceLayer], embedding, lm_head, g_final, dtype: str,
                 device="cuda:0"):
        self.ctx, self.layers, self.dtype, self.device = ctx, layers, dtype, device
        self.embedding = to_device(embedding, dtype, device)
        self.lm_head = to_device(lm_head, dtype, device)
        self.g_final = None if g_final is None else to_device(g_final, dtype, device)
        self.vocab, self.d = self.embedding.shape
        self.H = ctx.cfg.n_heads
        self.K = self.V = self.y = None

    def prefill(self, ids: torch.Tensor, N: int, kv_cap: int, keep_outputs: bool = True, wavefront: bool = False,
                chunk: int = 0):
        """ids [B, >= N] int32 on the device.  Runs positions 0..N-1 through every layer; returns the
        logits [B, vocab] (fp32) of position N-1.  Layer outputs stay in self.y[l] ([B, N, d]) and the
        caches in self.K[l], self.V[l] ([kv_cap, B, H, 64]).  wavefront: one rt_stack_prefill call (layers
        run concurrently, `chunk` positions apart) instead of one rt_layer_prefill per layer."""
        B = ids.shape[0]
        td = torch_dtype(self.dtype)
        x = torch.empty((B, N, self.d), dtype=td, device=self.device)
        self.ctx.rt_embed_rows(self.embedding, ids, 0, x)
        self.x0 = x
        self.K, self.V, self.y = [], [], []
        if wavefront:
            for _ in self.layers:
                self.y.append(torch.empty_like(x))
                self.K.append(torch.zeros((kv_cap, B, self.H, self.d // self.H), dtype=td, device=self.device))
                self.V.append(torch.zeros_like(self.K[-1]))
            self.ctx.rt_stack_prefill([lay.struct for lay in self.layers], x, self.y, self.K, self.V, chunk)
            x = self.y[-1]
        else:
            for lay in self.layers:
                y = torch.empty_like(x)
                K = torch.zeros((kv_cap, B, self.H, self.d // self.H), dtype=td, device=self.device)
                V = torch.zeros_like(K)
                self.ctx.rt_layer_prefill(lay.struct, x, y, K, V)
                self.K.append(K); self.V.append(V)
                if keep_outputs:
                    self.y.append(y)
                x = y
        self.last = x
        logits = torch.empty((B, self.vocab), dtype=torch.float32, device=self.device)
        self.ctx.rt_lm_head(self.lm_head, self.g_final, x[:, N - 1], x.stride(0), B, logits)
        return logits

    def decode_step(self, ids: torch.Tensor, t: int):
        """One position t (0-based) for all sequences: ids[:, t] is the input token.  Returns
        (logits [B, vocab] fp32, per-layer outputs [L, B, d])."""
        B = ids.shape[0]
        td = torch_dtype(self.dtype)
        L = len(self.layers)
        rows = torch.empty((L + 1, B, 1, self.d), dtype=td, device=self.device)
        self.ctx.rt_embed_rows(self.embedding, ids, t, rows[0])
        for l, lay in enumerate(self.layers):
            self.ctx.rt_decode_step(lay.struct, rows[l, :, 0], t, rows[l + 1, :, 0], self.K[l], self.V[l])
        logits = torch.empty((B, self.vocab), dtype=torch.float32, device=self.device)
        self.ctx.rt_lm_head(self.lm_head, self.g_final, rows[L], self.d, B, logits)
        return logits, rows[1:, :, 0]
