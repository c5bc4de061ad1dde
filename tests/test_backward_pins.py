"""Pins of the backward-pass oracle (oracle/rt_backward.py) against what is not that oracle (no GPU): central
differences of the pinned forward oracle, the Jacobian closed form of Theorem 4.1, the N = 1 closed form,
causality of the gradient, and a control that a dropped term is caught."""
import math

import numpy as np
import pytest
from scipy.special import erf

from paper_2604_21215_amd import inputs as gen
from oracle import rt_backward as bwd


def _small(seed, B=2, N=7, d=24, H=3, F=40, gains="random", w_std=0.3):
    li = gen.make_custom(seed, "f32", B, N, d, H, F, w_std=w_std, gains=gains)
    w = {k: v.astype(np.float64) for k, v in li.weights.items()}
    g = {k: v.astype(np.float64) for k, v in li.gains.items()}
    return li.x.astype(np.float64), w, g


def _loss(oracle, w, g, H, x, gy, gK, gV, **kw):
    y, K, V = oracle.Layer(w, H, gains=g, **kw).prefill(x)
    return float(np.sum(gy * y) + np.sum(gK * K) + np.sum(gV * V))


# ------------------------------------------------------------------------------------------
# B1  Central differences of the forward oracle (itself pinned) along random directions of every input.
#     L = <gy, y> + <gK, K> + <gV, V> with random gy, gK, gV, so every output channel is exercised.
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("alpha,scale,beta,eps", [(1.0, 1.0, 0.0, 1e-6), (0.6, 0.4, 8.0, 1e-2)])
def test_b1_central_differences_every_input_and_parameter(oracle, alpha, scale, beta, eps):
    x, w, g = _small(301)
    B, N, d = x.shape
    H = 3
    g["g_kv"] = g["g_kv"] * 1.1 + 0.05     # a gain of its own for RMS(z)
    rng = np.random.default_rng(5)
    gy, gK, gV = rng.standard_normal((B, N, d)), rng.standard_normal((N, B, H, d // H)), rng.standard_normal((N, B, H, d // H))
    kw = dict(alpha=alpha, attn_scale=scale, eps=eps, alibi_max_bias=beta)
    z = oracle.Layer(w, H, gains=g, **kw).prefill(x)[0]
    dx, dW, dG = bwd.layer_backward(w, H, x, z, gy, gK, gV, gains=g, **kw)
    h = 1e-6

    def directional(perturb):
        """(L(+h) - L(-h)) / 2h for a perturbation applied by perturb(sign * h) -> (x, w, g)."""
        xp, wp, gp = perturb(+h)
        xm, wm, gm = perturb(-h)
        return (_loss(oracle, wp, gp, H, xp, gy, gK, gV, **kw) - _loss(oracle, wm, gm, H, xm, gy, gK, gV, **kw)) / (2 * h)

    dirx = rng.standard_normal(x.shape)
    fd = directional(lambda e: (x + e * dirx, w, g))
    assert abs(fd - np.sum(dx * dirx)) <= 1e-6 * max(1.0, abs(fd)), ("x", fd, np.sum(dx * dirx))
    # one position at a time: a wrong term at a single position cannot hide in the sum
    for i in (0, N // 2, N - 1):
        di = np.zeros_like(x)
        di[:, i] = dirx[:, i]
        fd = directional(lambda e: (x + e * di, w, g))
        assert abs(fd - np.sum(dx * di)) <= 1e-6 * max(1.0, abs(fd)), ("x at", i)
    for name in bwd.PARAMS:
        dirw = rng.standard_normal(w[name].shape)
        fd = directional(lambda e: (x, {**w, name: w[name] + e * dirw}, g))
        an = np.sum(dW[name] * dirw)
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)), (name, fd, an)
    for name in bwd.GAINS:
        dirg = rng.standard_normal(g[name].shape)
        fd = directional(lambda e: (x, w, {**g, name: g[name] + e * dirg}))
        an = np.sum(dG[name] * dirg)
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)), (name, fd, an)


def test_b1_shared_gain_and_missing_output_projection(oracle):
    """g_kv absent (RMS(z) shares the gain of RMS(x)) and Wo absent (identity), as the forward oracle allows."""
    x, w, g = _small(302, N=5)
    H = 3
    w["Wo"] = None
    g = {k: v for k, v in g.items() if k != "g_kv"}
    rng = np.random.default_rng(6)
    gy = rng.standard_normal(x.shape)
    zero = np.zeros((x.shape[1], x.shape[0], H, x.shape[2] // H))
    z = oracle.Layer(w, H, gains=g).prefill(x)[0]
    dx, dW, dG = bwd.layer_backward(w, H, x, z, gy, gains=g)
    assert dW["Wo"] is None and dG["g_kv"] is None
    h = 1e-6
    dirg = rng.standard_normal(g["g_attn"].shape)
    fd = (_loss(oracle, w, {**g, "g_attn": g["g_attn"] + h * dirg}, H, x, gy, zero, zero)
          - _loss(oracle, w, {**g, "g_attn": g["g_attn"] - h * dirg}, H, x, gy, zero, zero)) / (2 * h)
    assert abs(fd - np.sum(dG["g_attn"] * dirg)) <= 1e-6 * max(1.0, abs(fd))
    dirx = rng.standard_normal(x.shape)
    fd = (_loss(oracle, w, g, H, x + h * dirx, gy, zero, zero) - _loss(oracle, w, g, H, x - h * dirx, gy, zero, zero)) / (2 * h)
    assert abs(fd - np.sum(dx * dirx)) <= 1e-6 * max(1.0, abs(fd))


# ------------------------------------------------------------------------------------------
# B2  A dropped term is caught: without the path through the persistent pair the x-gradient is wrong at
#     every position but the last (whose pair nobody attends).
# ------------------------------------------------------------------------------------------
def test_b2_planted_mistake_is_detected(oracle):
    x, w, g = _small(303, N=6)
    H = 3
    rng = np.random.default_rng(7)
    gy = rng.standard_normal(x.shape)
    z = oracle.Layer(w, H, gains=g).prefill(x)[0]
    good = bwd.layer_backward(w, H, x, z, gy, gains=g)[0]
    bad = bwd.layer_backward(w, H, x, z, gy, gains=g, drop_pair_gradient=True)[0]
    np.testing.assert_array_equal(good[:, -1], bad[:, -1])
    zero = np.zeros((x.shape[1], x.shape[0], H, x.shape[2] // H))
    h = 1e-6
    di = np.zeros_like(x)
    di[:, 1] = rng.standard_normal(x[:, 1].shape)
    fd = (_loss(oracle, w, g, H, x + h * di, gy, zero, zero) - _loss(oracle, w, g, H, x - h * di, gy, zero, zero)) / (2 * h)
    assert abs(fd - np.sum(good * di)) <= 1e-6 * max(1.0, abs(fd))
    assert abs(fd - np.sum(bad * di)) > 1e-3 * abs(fd)


# ------------------------------------------------------------------------------------------
# B3  Theorem 4.1: norm-free, zero queries (uniform attention), no MLP, Wo = I, single head:
#     dz_k / dx_1 = (1/k!) prod_{m=0}^{k-1} (alpha V + m I)   (for k >= 2; (I + alpha V) for k = 1).
#     The backward pass returns vector-Jacobian products: with gy = e_c at position k alone, dx_1 is row c of it.
# ------------------------------------------------------------------------------------------
def test_b3_theorem_4_1_jacobian(oracle):
    d, N, alpha = 5, 6, 0.7
    rng = np.random.default_rng(8)
    Vm = rng.standard_normal((d, d)) * 0.5
    w = {"Wq": np.zeros((d, d)), "Wk": rng.standard_normal((d, d)), "Wv": Vm, "Wo": None,
         "W1": rng.standard_normal((8, d)), "W2": np.zeros((d, 8))}
    x = rng.standard_normal((1, N, d))
    z = oracle.Layer(w, 1, alpha=alpha, norm_free=True).prefill(x)[0]
    for k in range(1, N + 1):
        J = np.eye(d)
        for m in range(k):
            J = J @ (alpha * Vm + m * np.eye(d))
        J = J / math.factorial(k) if k >= 2 else np.eye(d) + alpha * Vm
        for c in (0, d - 1):
            gy = np.zeros_like(x)
            gy[0, k - 1, c] = 1.0
            dx = bwd.layer_backward(w, 1, x, z, gy, alpha=alpha, norm_free=True)[0]
            np.testing.assert_allclose(dx[0, 0], J[c], rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------------------------------
# B4  N = 1: softmax over one term; the gradient is that of x -> h + alpha W2 gelu(W1 RMS(h)), h = x + alpha Wo Wv RMS(x)
#     written with dense Jacobians; Wq and Wk get no gradient from y.
# ------------------------------------------------------------------------------------------
def test_b4_single_position_closed_form(oracle):
    x, w, g = _small(304, B=1, N=1, gains="unit")
    H, eps = 3, 1e-3
    d = x.shape[2]
    gy = np.random.default_rng(9).standard_normal(x.shape)
    z = oracle.Layer(w, H, gains=g, eps=eps, alpha=0.8).prefill(x)[0]
    dx, dW, _ = bwd.layer_backward(w, H, x, z, gy, gains=g, eps=eps, alpha=0.8)

    def rms_jac(u):
        r = 1.0 / math.sqrt(np.mean(u * u) + eps)
        return r * np.eye(d) - r ** 3 * np.outer(u, u) / d

    x1 = x[0, 0]
    A = 0.8 * w["Wo"] @ w["Wv"]
    h = x1 + A @ (x1 / math.sqrt(np.mean(x1 * x1) + eps))
    Jh = np.eye(d) + A @ rms_jac(x1)
    m = h / math.sqrt(np.mean(h * h) + eps)
    pre = w["W1"] @ m
    gp = 0.5 * (1.0 + erf(pre / math.sqrt(2.0))) + pre * np.exp(-0.5 * pre * pre) / math.sqrt(2.0 * math.pi)
    Jz = (np.eye(d) + 0.8 * w["W2"] @ (gp[:, None] * w["W1"]) @ rms_jac(h)) @ Jh
    np.testing.assert_allclose(dx[0, 0], Jz.T @ gy[0, 0], rtol=1e-10, atol=1e-12)
    assert np.abs(dW["Wq"]).max() == 0.0


# ------------------------------------------------------------------------------------------
# B5  Causality of the gradient: an upstream gradient on outputs <= t alone gives no gradient to inputs > t, and
#     adding upstream gradient on later outputs leaves nothing of that statement changed for the earlier loss.
# ------------------------------------------------------------------------------------------
def test_b5_gradient_is_causal(oracle):
    x, w, g = _small(305, N=8)
    H, t = 3, 4
    rng = np.random.default_rng(10)
    gy = rng.standard_normal(x.shape)
    gy[:, t + 1:] = 0.0
    z = oracle.Layer(w, H, gains=g).prefill(x)[0]
    dx = bwd.layer_backward(w, H, x, z, gy, gains=g)[0]
    assert np.abs(dx[:, t + 1:]).max() == 0.0
    assert np.abs(dx[:, :t + 1]).min() > 0.0
