"""Shared helpers of the GPU parity tests: run the oracle and the HIP path on the same buffers and
reduce the differences to error curves over position."""
from __future__ import annotations

import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}
# The attention + MLP branch y - x alone (y = x + branch hides an error of the branch behind the untouched x): held to
# the same norm-wise bound as y, K and V, measured against the norm of the exact branch.
BRANCH_TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_err_rows(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Norm-wise relative error over the last axis."""
    num = np.linalg.norm(got - ref, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    return num / np.maximum(den, 1e-30)


def error_curves(x, ref, got):
    """ref, got = (y [B,N,d], K [N,B,H,dh], V [N,B,H,dh]) as float64.  Returns dict name -> curve over t
    (max over batch rows, and over heads for K and V) plus the attention+MLP branch error (y - x)."""
    y_r, K_r, V_r = ref
    y_g, K_g, V_g = got
    N = y_r.shape[1]
    out = {
        "y": rel_err_rows(y_g, y_r).max(axis=0),
        "K": rel_err_rows(K_g[:N], K_r[:N]).reshape(N, -1).max(axis=1),
        "V": rel_err_rows(V_g[:N], V_r[:N]).reshape(N, -1).max(axis=1),
        "branch": rel_err_rows(y_g - x, y_r - x).max(axis=0),
    }
    return out


def summarize(curves) -> str:
    parts = []
    for k, c in curves.items():
        n = len(c)
        qs = [c[: max(1, n // 4)].max(), c[n // 4: max(n // 4 + 1, n // 2)].max() if n > 1 else c.max(),
              c[n // 2: max(n // 2 + 1, 3 * n // 4)].max() if n > 1 else c.max(), c[3 * n // 4:].max() if n > 1 else c.max()]
        parts.append("%s max=%.3e (quarters %s)" % (k, c.max(), " ".join("%.1e" % q for q in qs)))
    return "; ".join(parts)


def oracle_layer(oracle, li, H, **kw):
    w = {k: v.astype(np.float64) for k, v in li.weights.items()}
    g = {k: v.astype(np.float64) for k, v in li.gains.items()}
    return oracle.Layer(w, H, gains=g, **kw)
