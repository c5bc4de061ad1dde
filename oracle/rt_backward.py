"""fp64 CPU oracle of the RT layer's backward pass -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; nothing here is shared with the
HIP library.  Plain numpy, one position at a time, no tiling, direct softmax.

What it computes has a plain definition: for the layer map (x, parameters) -> (y, K, V) of Sec. 2.2 and a linear
functional  L = <gy, y> + <gK, K> + <gV, V>,  the gradients of L with respect to x and to every parameter.  It is
written out as reverse-mode differentiation of the definition in the order Sec. 6.4 ("The backward pass") gives:

  * the positions are visited in reverse.  Position i first completes the gradient of its output z_i: the upstream
    gy_i plus what arrives through its persistent pair k_i = qkRMS(Wk RMS(z_i)), v_i = Wv RMS(z_i), whose gradients
    (dK_i, dV_i) have by then been accumulated from every later position's attention;
  * that gradient goes back through  z_i = h_i + alpha W2 gelu(W1 RMS(h_i)),  h_i = x_i + alpha Wo c_i  to the
    attention output c_i, and through the softmax of position i it ADDS to dK_j, dV_j of the earlier positions j < i
    - the only quantity the reverse loop has to carry from one position to the next;
  * the gradients with respect to q_i, the temporary pair, x (through RMS and the three projections) and all
    parameters impose no such dependency: they are collected per position and reduced after the loop.

Forward intermediates are recomputed from (x, z) as Sec. 6.1 ("Activation checkpointing") describes: with z = the
layer's output given, every persistent pair is rebuilt from RMS(z) at once, and position i's logits, softmax weights,
attention output, h_i and MLP pre-activations follow from x_i and the pairs of positions < i.

Readings (the same as the forward oracle's): RMS(u) = g u / sqrt(mean(u^2) + eps); qkRMS the same per head;
exact (erf) GELU; logits attn_scale <k, q> minus the ALiBi bias slope_h (i - j); alpha on both branches.

Pinned by tests/test_backward_pins.py: central differences of the pinned forward oracle (every input and parameter),
the Jacobian closed form of Theorem 4.1, the N = 1 closed form, causality of the gradient, and a planted-mistake control.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf

PARAMS = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")
GAINS = ("g_attn", "g_mlp", "g_kv", "g_q", "g_k")


def _gelu(p):
    return 0.5 * p * (1.0 + erf(p / math.sqrt(2.0)))


def _gelu_grad(p):
    return 0.5 * (1.0 + erf(p / math.sqrt(2.0))) + p * np.exp(-0.5 * p * p) / math.sqrt(2.0 * math.pi)


class _Norm:
    """y = g u / sqrt(mean(u^2) + eps) over the last axis (identity when norm_free), with its transpose Jacobian."""

    def __init__(self, u, g, eps, norm_free):
        self.nf = norm_free
        self.g = None if g is None else np.asarray(g, dtype=np.float64)
        if norm_free:
            self.y = u
            return
        self.D = u.shape[-1]
        self.r = 1.0 / np.sqrt(np.mean(u * u, axis=-1, keepdims=True) + eps)
        self.unit = u * self.r                      # normalised, before the gain
        self.y = self.unit if self.g is None else self.unit * self.g

    def backward(self, dy):
        """Returns (du, dg); dg summed over every leading axis (None without a gain or when norm_free)."""
        if self.nf:
            return dy, None
        w = dy if self.g is None else dy * self.g
        du = self.r * (w - self.unit * np.sum(self.unit * w, axis=-1, keepdims=True) / self.D)
        dg = None
        if self.g is not None:
            dg = (dy * self.unit).reshape(-1, *self.g.shape).sum(axis=0)
        return du, dg


def layer_backward(weights, H, x, z, gy, gK=None, gV=None, *, gains=None, alpha=1.0, attn_scale=1.0, eps=1e-6,
                   norm_free=False, alibi_max_bias=0.0, drop_pair_gradient=False):
    """Gradients of L = <gy, y> + <gK, K> + <gV, V> for one RT layer.

    weights: dict Wq, Wk, Wv [d,d], Wo [d,d] or None (identity), W1 [F,d], W2 [d,F];  gains: dict or None (ones).
    x, z, gy: [B, N, d] (z = the layer's output for x, e.g. from oracle.rt_oracle.Layer.prefill);
    gK, gV: [N, B, H, dh] or None (zero).
    drop_pair_gradient: test control only - leaves out the term that reaches z_i through its persistent pair.
    Returns (dx [B,N,d], dW dict over the six matrices, dG dict over the five gain vectors)."""
    x, z, gy = (np.asarray(a, dtype=np.float64) for a in (x, z, gy))
    B, N, d = x.shape
    dh = d // H
    W = {k: (None if weights.get(k) is None else np.asarray(weights[k], dtype=np.float64)) for k in PARAMS}
    g = {k: None for k in GAINS}
    for k, v in (gains or {}).items():
        g[k] = None if v is None else np.asarray(v, dtype=np.float64)
    if g["g_kv"] is None:
        g["g_kv"] = g["g_attn"]
    shared_kv_gain = gains is None or gains.get("g_kv") is None
    gq = None if g["g_q"] is None else g["g_q"].reshape(H, dh)
    gk = None if g["g_k"] is None else g["g_k"].reshape(H, dh)
    slopes = np.array([2.0 ** (-alibi_max_bias * (h + 1) / H) if alibi_max_bias > 0 else 0.0 for h in range(H)])

    # ---- recompute (Sec. 6.1): everything that depends on x or z alone, all positions at once
    n_x = _Norm(x, g["g_attn"], eps, norm_free)                                   # RMS(x_i)
    q_n = _Norm((n_x.y @ W["Wq"].T).reshape(B, N, H, dh), gq, eps, norm_free)     # q_i
    kt_n = _Norm((n_x.y @ W["Wk"].T).reshape(B, N, H, dh), gk, eps, norm_free)    # temporary key
    vt = (n_x.y @ W["Wv"].T).reshape(B, N, H, dh)                                 # temporary value
    n_z = _Norm(z, g["g_kv"], eps, norm_free)                                     # RMS(z_i)
    k_n = _Norm((n_z.y @ W["Wk"].T).reshape(B, N, H, dh), gk, eps, norm_free)     # persistent key
    v_p = (n_z.y @ W["Wv"].T).reshape(B, N, H, dh)                                # persistent value
    q, kt, k_p = q_n.y, kt_n.y, k_n.y

    dK = np.zeros((B, N, H, dh)) if gK is None else np.asarray(gK, dtype=np.float64).transpose(1, 0, 2, 3).copy()
    dV = np.zeros((B, N, H, dh)) if gV is None else np.asarray(gV, dtype=np.float64).transpose(1, 0, 2, 3).copy()
    dq = np.zeros((B, N, H, dh))
    dkt = np.zeros((B, N, H, dh))
    dvt = np.zeros((B, N, H, dh))
    dh_all = np.zeros((B, N, d))          # gradient of h_i (reaches x_i directly through the residual)
    dz_rms = np.zeros((B, N, d))          # gradient of RMS(z_i) (persistent-pair path), kept for the parameter sums
    dW = {k: (None if W[k] is None else np.zeros_like(W[k])) for k in PARAMS}
    dG = {k: (None if g[k] is None or norm_free else np.zeros_like(g[k])) for k in GAINS}

    # ---- the reverse loop (Sec. 6.4): carries only dK, dV
    for i in range(N - 1, -1, -1):
        # forward of position i (recomputed): logits over persistent pairs j < i and the own temporary pair
        S = attn_scale * np.einsum("bjhc,bhc->bhj", k_p[:, :i], q[:, i])
        S = S - slopes[None, :, None] * (i - np.arange(i))[None, None, :]
        s_own = attn_scale * np.sum(kt[:, i] * q[:, i], axis=-1)                   # [B, H]
        mx = np.maximum(S.max(axis=-1) if i else -np.inf, s_own)
        E, e_own = np.exp(S - mx[..., None]), np.exp(s_own - mx)
        den = E.sum(axis=-1) + e_own
        P, p_own = E / den[..., None], e_own / den
        c = np.einsum("bhj,bjhc->bhc", P, v_p[:, :i]) + p_own[..., None] * vt[:, i]
        cat = c.reshape(B, d)
        a = cat if W["Wo"] is None else cat @ W["Wo"].T
        h_i = x[:, i] + alpha * a
        m_n = _Norm(h_i, g["g_mlp"], eps, norm_free)
        pre = m_n.y @ W["W1"].T
        act = _gelu(pre)

        # gradient of z_i: upstream plus the path through the persistent pair of position i
        Gz = gy[:, i].copy()
        dkraw, dgk_i = k_n_backward(k_n, i, dK[:, i])
        d_rz = dkraw.reshape(B, d) @ W["Wk"] + dV[:, i].reshape(B, d) @ W["Wv"]
        dz_rms[:, i] = d_rz
        if not drop_pair_gradient:
            Gz = Gz + norm_rows_backward(n_z, i, d_rz)
        dW["Wk"] += dkraw.reshape(B, d).T @ n_z.y[:, i]
        dW["Wv"] += dV[:, i].reshape(B, d).T @ n_z.y[:, i]
        if dG["g_k"] is not None and dgk_i is not None:
            dG["g_k"] += dgk_i.reshape(-1)

        # z_i = h_i + alpha W2 gelu(W1 RMS(h_i))
        dmo = alpha * Gz
        dW["W2"] += dmo.T @ act
        dpre = (dmo @ W["W2"]) * _gelu_grad(pre)
        dW["W1"] += dpre.T @ m_n.y
        dm, dg_mlp = m_n.backward(dpre @ W["W1"])
        if dG["g_mlp"] is not None and dg_mlp is not None:
            dG["g_mlp"] += dg_mlp
        d_h = Gz + dm
        dh_all[:, i] = d_h
        # h_i = x_i + alpha Wo c_i
        da = alpha * d_h
        if W["Wo"] is None:
            dc = da.reshape(B, H, dh)
        else:
            dW["Wo"] += da.T @ cat
            dc = (da @ W["Wo"]).reshape(B, H, dh)
        # softmax attention of position i
        dP = np.einsum("bhc,bjhc->bhj", dc, v_p[:, :i])
        dp_own = np.sum(dc * vt[:, i], axis=-1)
        Dsum = np.sum(P * dP, axis=-1) + p_own * dp_own
        dS = P * (dP - Dsum[..., None])
        ds_own = p_own * (dp_own - Dsum)
        dV[:, :i] += np.einsum("bhj,bhc->bjhc", P, dc)                              # carried to earlier positions
        dK[:, :i] += attn_scale * np.einsum("bhj,bhc->bjhc", dS, q[:, i])           # carried to earlier positions
        dvt[:, i] = p_own[..., None] * dc
        dkt[:, i] = attn_scale * ds_own[..., None] * q[:, i]
        dq[:, i] = attn_scale * (np.einsum("bhj,bjhc->bhc", dS, k_p[:, :i]) + ds_own[..., None] * kt[:, i])

    # ---- after the loop, batched over all positions: q, the temporary pairs, x and the remaining parameter sums
    dq_raw, dgq = q_n.backward(dq)
    dkt_raw, dgk_t = kt_n.backward(dkt)
    M = B * N
    dn = dq_raw.reshape(M, d) @ W["Wq"] + dkt_raw.reshape(M, d) @ W["Wk"] + dvt.reshape(M, d) @ W["Wv"]
    nx2 = n_x.y.reshape(M, d)
    dW["Wq"] += dq_raw.reshape(M, d).T @ nx2
    dW["Wk"] += dkt_raw.reshape(M, d).T @ nx2
    dW["Wv"] += dvt.reshape(M, d).T @ nx2
    dx_n, dg_attn = n_x.backward(dn.reshape(B, N, d))
    dx = dh_all + dx_n
    if not norm_free:
        if dG["g_q"] is not None and dgq is not None:
            dG["g_q"] += dgq.reshape(-1)
        if dG["g_k"] is not None and dgk_t is not None:
            dG["g_k"] += dgk_t.reshape(-1)
        if dG["g_attn"] is not None and dg_attn is not None:
            dG["g_attn"] += dg_attn
        # gain of RMS(z): the persistent-pair path
        if g["g_kv"] is not None:
            dg_kv = (dz_rms * n_z.unit).reshape(M, d).sum(axis=0)
            if shared_kv_gain:
                if dG["g_attn"] is not None:
                    dG["g_attn"] += dg_kv
                dG["g_kv"] = None
            else:
                dG["g_kv"] += dg_kv
    return dx, dW, dG


def k_n_backward(k_n, i, dk_i):
    """Transpose Jacobian of the per-head normalisation of the persistent key of position i: (d raw key, d gain)."""
    if k_n.nf:
        return dk_i, None
    w = dk_i if k_n.g is None else dk_i * k_n.g
    unit, r = k_n.unit[:, i], k_n.r[:, i]
    du = r * (w - unit * np.sum(unit * w, axis=-1, keepdims=True) / k_n.D)
    dg = None if k_n.g is None else (dk_i * unit).sum(axis=0)
    return du, dg


def norm_rows_backward(n_z, i, dy):
    """Transpose Jacobian of RMS(z_i) for the rows of position i (gain gradient handled by the caller)."""
    if n_z.nf:
        return dy
    w = dy if n_z.g is None else dy * n_z.g
    unit, r = n_z.unit[:, i], n_z.r[:, i]
    return r * (w - unit * np.sum(unit * w, axis=-1, keepdims=True) / n_z.D)
