"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Every check compares the oracle with something that is not the oracle: closed forms written
with dense numpy algebra, theorems of the paper, structural invariants, or worked examples.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import erf

from paper_2604_21215_amd import inputs as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _gelu(u):
    return 0.5 * u * (1.0 + erf(u / math.sqrt(2.0)))


def _rms(x, g=None, eps=0.0):
    r = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return r if g is None else r * g


def _small(seed, B=2, N=9, d=16, H=2, F=32, gains="random", w_std=0.3):
    li = gen.make_custom(seed, "f32", B, N, d, H, F, w_std=w_std, gains=gains)
    w = {k: v.astype(np.float64) for k, v in li.weights.items()}
    g = {k: v.astype(np.float64) for k, v in li.gains.items()}
    return li.x.astype(np.float64), w, g


# ------------------------------------------------------------------------------------------
# P1  N = 1: the softmax has a single term, so a_1 = Wo Wv RMS(x_1) whatever Wq, Wk are
#     (Sec. 2.2, displays for a_i and z_i).
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("alpha,eps,scale", [(1.0, 0.0, 1.0), (0.5, 0.1, 0.37)])
def test_p1_single_position_closed_form(oracle, alpha, eps, scale):
    x, w, g = _small(11, B=3, N=1)
    H, d = 2, 16
    lay = oracle.Layer(w, H, gains=g, alpha=alpha, eps=eps, attn_scale=scale)
    y, K, V = lay.prefill(x)
    for b in range(3):
        x1 = x[b, 0]
        n = _rms(x1, g["g_attn"], eps)
        a = w["Wo"] @ (w["Wv"] @ n)
        h = x1 + alpha * a
        z = h + alpha * (w["W2"] @ _gelu(w["W1"] @ _rms(h, g["g_mlp"], eps)))
        np.testing.assert_allclose(y[b, 0], z, rtol=1e-12, atol=1e-13)
        r = _rms(z, g["g_kv"], eps)
        k = (w["Wk"] @ r).reshape(H, d // H)
        k = _rms(k, g["g_k"].reshape(H, -1), eps)
        np.testing.assert_allclose(K[0, b], k, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(V[0, b], (w["Wv"] @ r).reshape(H, -1), rtol=1e-12, atol=1e-13)
    # Wq, Wk do not matter at N = 1 for y and V
    w2 = dict(w)
    w2["Wq"] = w["Wq"][::-1].copy()
    y2, _, V2 = oracle.Layer(w2, H, gains=g, alpha=alpha, eps=eps, attn_scale=scale).prefill(x)
    np.testing.assert_array_equal(y, y2)
    np.testing.assert_array_equal(V, V2)


# ------------------------------------------------------------------------------------------
# P2  Causality: inputs after t never reach outputs at or before t.
# ------------------------------------------------------------------------------------------
def test_p2_causality_bit_identical(oracle):
    x, w, g = _small(12, B=2, N=12)
    lay = oracle.Layer(w, 2, gains=g)
    y, K, V = lay.prefill(x)
    t = 7
    x2 = x.copy()
    x2[:, t:] += 3.0
    y2, K2, V2 = lay.prefill(x2)
    np.testing.assert_array_equal(y[:, :t], y2[:, :t])
    np.testing.assert_array_equal(K[:t], K2[:t])
    np.testing.assert_array_equal(V[:t], V2[:t])
    assert np.abs(y[:, t:] - y2[:, t:]).max() > 1e-3


# ------------------------------------------------------------------------------------------
# P3  Brute force: re-evaluate the whole prefix from scratch for every t, and an independent
#     dense re-statement of the recurrence in numpy for tiny N.
# ------------------------------------------------------------------------------------------
def _rt_numpy(x, w, g, H, alpha=1.0, eps=0.0, scale=1.0, alibi=0.0):
    """One sequence [N, d]; nothing cached except the outputs the definition itself refers to.
    alibi = beta: logits get -2^(-beta (h+1)/H) (i - j) for the persistent key of position j (Press et al.)."""
    N, d = x.shape
    dh = d // H
    gq, gk = g["g_q"].reshape(H, dh), g["g_k"].reshape(H, dh)
    z = np.zeros((N, d))
    for i in range(N):
        n = _rms(x[i], g["g_attn"], eps)
        q = _rms((w["Wq"] @ n).reshape(H, dh), gq, eps)
        kt = _rms((w["Wk"] @ n).reshape(H, dh), gk, eps)
        vt = (w["Wv"] @ n).reshape(H, dh)
        # persistent pairs of all earlier positions, recomputed from their outputs
        R = _rms(z[:i], g["g_kv"], eps)
        Kp = _rms((R @ w["Wk"].T).reshape(i, H, dh), gk, eps)
        Vp = (R @ w["Wv"].T).reshape(i, H, dh)
        heads = []
        for h in range(H):
            keys = np.vstack([Kp[:, h], kt[h][None]])
            vals = np.vstack([Vp[:, h], vt[h][None]])
            s = scale * (keys @ q[h])
            if alibi:
                s = s - 2.0 ** (-alibi * (h + 1) / H) * (i - np.arange(i + 1))   # last entry: the temporary pair, distance 0
            p = np.exp(s - s.max())
            heads.append((p / p.sum()) @ vals)
        a = w["Wo"] @ np.concatenate(heads)
        hdd = x[i] + alpha * a
        z[i] = hdd + alpha * (w["W2"] @ _gelu(w["W1"] @ _rms(hdd, g["g_mlp"], eps)))
    return z


def test_p3_bruteforce_prefix_and_dense_restatement(oracle):
    x, w, g = _small(13, B=2, N=10)
    lay = oracle.Layer(w, 2, gains=g, alpha=0.7, eps=1e-6, attn_scale=0.5)
    y, K, V = lay.prefill(x)
    for t in range(1, 11):
        yt, Kt, Vt = lay.prefill(x[:, :t])
        np.testing.assert_array_equal(yt[:, t - 1], y[:, t - 1])
        np.testing.assert_array_equal(Kt[t - 1], K[t - 1])
    for b in range(2):
        z = _rt_numpy(x[b], w, g, 2, alpha=0.7, eps=1e-6, scale=0.5)
        np.testing.assert_allclose(y[b], z, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------------------------------
# P4  Fixed point (Sec. 6.1, "Activation Checkpointing"): given z, rebuild all persistent pairs
#     at once, run ordinary masked attention with the temporary pair on the diagonal and the MLP
#     in parallel; the result must reproduce z.  By induction on position the fixed point is
#     unique, so zero residual means z is the layer's output.
# ------------------------------------------------------------------------------------------
def _parallel_recompute(x, z, w, g, H, alpha, eps, scale, alibi=0.0):
    N, d = x.shape
    dh = d // H
    gq, gk = g["g_q"].reshape(H, dh), g["g_k"].reshape(H, dh)
    n = _rms(x, g["g_attn"], eps)
    Q = _rms((n @ w["Wq"].T).reshape(N, H, dh), gq, eps)
    Kt = _rms((n @ w["Wk"].T).reshape(N, H, dh), gk, eps)
    Vt = (n @ w["Wv"].T).reshape(N, H, dh)
    r = _rms(z, g["g_kv"], eps)
    Kp = _rms((r @ w["Wk"].T).reshape(N, H, dh), gk, eps)
    Vp = (r @ w["Wv"].T).reshape(N, H, dh)
    cat = np.zeros((N, H, dh))
    for h in range(H):
        S = scale * (Q[:, h] @ Kp[:, h].T)                      # [i, j]
        if alibi:
            S = S - 2.0 ** (-alibi * (h + 1) / H) * (np.arange(N)[:, None] - np.arange(N)[None, :])
        S[np.triu_indices(N, 0)] = -np.inf                      # strictly lower triangle is visible
        S[np.arange(N), np.arange(N)] = scale * np.sum(Q[:, h] * Kt[:, h], axis=1)
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        diag = np.diag(P).copy()
        np.fill_diagonal(P, 0.0)
        cat[:, h] = P @ Vp[:, h] + diag[:, None] * Vt[:, h]
    a = cat.reshape(N, d) @ w["Wo"].T
    hdd = x + alpha * a
    return hdd + alpha * (_gelu(_rms(hdd, g["g_mlp"], eps) @ w["W1"].T) @ w["W2"].T), Kp, Vp


@pytest.mark.parametrize("N,scale", [(33, 1.0), (20, 0.125)])
def test_p4_fixed_point_parallel_recompute(oracle, N, scale):
    x, w, g = _small(14, B=2, N=N, d=24, H=3, F=40)
    alpha, eps = 0.6, 1e-5
    y, K, V = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale).prefill(x)
    for b in range(2):
        z2, Kp, Vp = _parallel_recompute(x[b], y[b], w, g, 3, alpha, eps, scale)
        np.testing.assert_allclose(z2, y[b], rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(K[:, b], Kp, rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(V[:, b], Vp, rtol=1e-10, atol=1e-11)


@pytest.mark.parametrize("beta", [0.0, 8.0])
def test_p4_oracle_recompute(oracle, beta):
    """oracle.Layer.recompute (the layer with its output given, Sec. 6.1): (1) the output of the token-by-token recurrence
    is its fixed point, with the same persistent pairs; (2) for an arbitrary z (not a fixed point) it agrees with the
    independent dense restatement above; (3) a perturbed z does not reproduce itself."""
    x, w, g = _small(16, B=2, N=21, d=24, H=3, F=40)
    alpha, eps, scale = 0.6, 1e-5, 0.5
    lay = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale, alibi_max_bias=beta)
    y, K, V = lay.prefill(x)
    y2, K2, V2 = lay.recompute(x, y)
    np.testing.assert_allclose(y2, y, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(K2, K, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(V2, V, rtol=1e-10, atol=1e-11)
    z = y + 0.3 * gen.normal(16, 9, y.shape, 1.0).astype(np.float64)
    y3, K3, V3 = lay.recompute(x, z)
    assert np.abs(y3 - z).max() > 1e-2
    for b in range(2):
        ref, Kp, Vp = _parallel_recompute(x[b], z[b], w, g, 3, alpha, eps, scale, alibi=beta)
        np.testing.assert_allclose(y3[b], ref, rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(K3[:, b], Kp, rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(V3[:, b], Vp, rtol=1e-10, atol=1e-11)


def test_p4_fixed_point_detects_planted_mistakes(oracle):
    """The residual is not vacuous: a wrong sign / dropped term / transposed matrix shows up."""
    x, w, g = _small(15, B=1, N=12)
    y, _, _ = oracle.Layer(w, 2, gains=g, eps=0.0).prefill(x)
    ok, _, _ = _parallel_recompute(x[0], y[0], w, g, 2, 1.0, 0.0, 1.0)
    assert np.abs(ok - y[0]).max() < 1e-10
    wt = dict(w)
    wt["Wo"] = w["Wo"].T.copy()
    bad, _, _ = _parallel_recompute(x[0], y[0], wt, g, 2, 1.0, 0.0, 1.0)
    assert np.abs(bad - y[0]).max() > 1e-3
    yT, _, _ = oracle.Layer(w, 2, gains=g, eps=0.0).transformer(x)   # KV from the input, not from z
    badT, _, _ = _parallel_recompute(x[0], yT[0], w, g, 2, 1.0, 0.0, 1.0)
    assert np.abs(badT - yT[0]).max() > 1e-3


# ------------------------------------------------------------------------------------------
# Transformer oracle against the textbook dense causal layer (Sec. 2.1).
# ------------------------------------------------------------------------------------------
def test_transformer_layer_matches_dense_causal_attention(oracle):
    x, w, g = _small(16, B=2, N=14)
    H, d = 2, 16
    dh = d // H
    alpha, eps, scale = 0.8, 1e-6, 0.4
    y, _, _ = oracle.Layer(w, H, gains=g, alpha=alpha, eps=eps, attn_scale=scale).transformer(x)
    for b in range(2):
        n = _rms(x[b], g["g_attn"], eps)
        Q = _rms((n @ w["Wq"].T).reshape(-1, H, dh), g["g_q"].reshape(H, dh), eps)
        Kk = _rms((n @ w["Wk"].T).reshape(-1, H, dh), g["g_k"].reshape(H, dh), eps)
        Vv = (n @ w["Wv"].T).reshape(-1, H, dh)
        cat = np.zeros_like(Vv)
        for h in range(H):
            S = scale * Q[:, h] @ Kk[:, h].T
            S[np.triu_indices(14, 1)] = -np.inf
            P = np.exp(S - S.max(axis=1, keepdims=True))
            cat[:, h] = (P / P.sum(axis=1, keepdims=True)) @ Vv[:, h]
        hdd = x[b] + alpha * cat.reshape(-1, d) @ w["Wo"].T
        ref = hdd + alpha * (_gelu(_rms(hdd, g["g_mlp"], eps) @ w["W1"].T) @ w["W2"].T)
        np.testing.assert_allclose(y[b], ref, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------------------------------
# P5  Appendix A: a width-3d' norm-free RT layer reproduces a width-d' norm-free Transformer
#     layer exactly (carry / live / scratch blocks), attention weights included, and stacks
#     after swapping carry and live.
# ------------------------------------------------------------------------------------------
def _emulation_layer(oracle, wT, mlpT, dp):
    Z = np.zeros((dp, dp))
    Qb = np.block([[wT["Wq"], Z, Z], [Z, Z, Z], [Z, Z, Z]])
    Kb = np.block([[wT["Wk"], Z, Z], [Z, Z, Z], [Z, Z, Z]])
    Vb = np.block([[Z, Z, Z], [Z, Z, Z], [wT["Wv"], Z, Z]])

    def mlp(u):
        c, l, s = u[:dp], u[dp:2 * dp], u[2 * dp:]
        return np.concatenate([np.zeros(dp), c + s + mlpT(c + s) - l, -s])

    return oracle.Layer({"Wq": Qb, "Wk": Kb, "Wv": Vb, "Wo": None}, 1, norm_free=True, alpha=1.0, mlp=mlp)


def test_p5_transformer_emulation_exact(oracle):
    dp, N, B = 5, 11, 2
    rng_w = [gen.normal(21, 50 + i, (dp, dp), 0.6).astype(np.float64) for i in range(8)]
    M1 = gen.normal(21, 70, (7, dp), 0.7).astype(np.float64)
    M2 = gen.normal(21, 71, (dp, 7), 0.7).astype(np.float64)
    xT = gen.activations(21, 1, B, N, dp).astype(np.float64)
    junk = gen.activations(21, 2, B, N, dp).astype(np.float64)     # the '*' block may hold anything

    def mlpT(u):
        return M2 @ np.tanh(M1 @ u)

    layersT = [{"Wq": rng_w[0], "Wk": rng_w[1], "Wv": rng_w[2], "Wo": None},
               {"Wq": rng_w[3], "Wk": rng_w[4], "Wv": rng_w[5], "Wo": None}]
    # layer 1
    T1 = oracle.Layer(layersT[0], 1, norm_free=True, mlp=mlpT)
    yT1, KT1, VT1, awT1 = T1.transformer(xT, want_attw=True)
    R1 = _emulation_layer(oracle, layersT[0], mlpT, dp)
    x1 = np.concatenate([xT, junk, np.zeros_like(xT)], axis=2)
    z1, K1, V1, aw1 = R1.prefill(x1, want_attw=True)
    np.testing.assert_allclose(z1[..., :dp], xT, rtol=0, atol=1e-12)          # carry kept
    np.testing.assert_allclose(z1[..., dp:2 * dp], yT1, rtol=1e-11, atol=1e-11)  # live = Transformer output
    np.testing.assert_allclose(z1[..., 2 * dp:], 0.0, atol=1e-12)             # scratch cancelled
    np.testing.assert_allclose(aw1, awT1, rtol=1e-11, atol=1e-13)             # (i) attention weights match
    np.testing.assert_allclose(K1[..., :dp], KT1, rtol=1e-11, atol=1e-12)     # persistent = embedded pairs
    np.testing.assert_allclose(K1[..., dp:], 0.0, atol=1e-12)
    np.testing.assert_allclose(V1[..., 2 * dp:], VT1, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(V1[..., :2 * dp], 0.0, atol=1e-12)
    # layer 2 after the carry <-> live swap
    T2 = oracle.Layer(layersT[1], 1, norm_free=True, mlp=mlpT)
    yT2, _, _, awT2 = T2.transformer(yT1, want_attw=True)
    x2 = np.concatenate([z1[..., dp:2 * dp], z1[..., :dp], z1[..., 2 * dp:]], axis=2)
    z2, _, _, aw2 = _emulation_layer(oracle, layersT[1], mlpT, dp).prefill(x2, want_attw=True)
    np.testing.assert_allclose(z2[..., dp:2 * dp], yT2, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(aw2, awT2, rtol=1e-10, atol=1e-12)
    # and the RT layer is not a Transformer in general: with K, V reading the whole vector it differs
    Rg = oracle.Layer({"Wq": np.eye(3 * dp), "Wk": np.eye(3 * dp), "Wv": np.eye(3 * dp), "Wo": None}, 1,
                      norm_free=True, mlp=lambda u: np.tanh(u))
    zr, _, _ = Rg.prefill(x1 * 0.3)
    zt, _, _ = Rg.transformer(x1 * 0.3)
    assert np.abs(zr[:, 1:] - zt[:, 1:]).max() > 1e-3
    np.testing.assert_allclose(zr[:, 0], zt[:, 0], rtol=1e-12, atol=1e-12)    # first position has no past


# ------------------------------------------------------------------------------------------
# P6  Theorem 4.1: uniform attention (Wq = 0), no norms, no MLP, single head.
#     z_k = x_k + (alpha/k) (V x_k + V sum_{j<k} z_j);  dz_k/dx_1 = (1/k!) prod_{m<k} (alpha V + m I)
#     = (1/k!) sum_r [k r] alpha^r V^r  for k >= 2, and I + alpha V for k = 1.
# ------------------------------------------------------------------------------------------
def _stirling_table():
    rows = []
    with open(os.path.join(GOLDEN, "stirling_first_kind.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(v) for v in line.split()])
    return rows


def test_p6_uniform_attention_jacobian_closed_form(oracle):
    d, N, alpha = 4, 7, 0.8
    Vm = gen.normal(31, 1, (d, d), 0.5).astype(np.float64)
    Z = np.zeros((d, d))
    w = {"Wq": Z, "Wk": gen.normal(31, 2, (d, d), 0.5).astype(np.float64), "Wv": Vm, "Wo": None,
         "W1": np.zeros((3, d)), "W2": np.zeros((d, 3))}
    lay = oracle.Layer(w, 1, norm_free=True, alpha=alpha)
    st = _stirling_table()
    aV = alpha * Vm
    for j in range(d):
        x = np.zeros((1, N, d))
        x[0, 0, j] = 1.0
        y, _, _ = lay.prefill(x)
        np.testing.assert_allclose(y[0, 0], (np.eye(d) + aV)[:, j], rtol=1e-13, atol=1e-14)
        for k in range(2, N + 1):
            prod = np.eye(d)
            for m in range(k):
                prod = prod @ (aV + m * np.eye(d))
            fk = prod / math.factorial(k)
            np.testing.assert_allclose(y[0, k - 1], fk[:, j], rtol=1e-11, atol=1e-13)
            series = sum(st[k - 1][r - 1] * np.linalg.matrix_power(aV, r) for r in range(1, k + 1))
            np.testing.assert_allclose(y[0, k - 1], (series / math.factorial(k))[:, j], rtol=1e-10, atol=1e-13)
    # the recurrence itself, for a generic input
    x = gen.activations(31, 3, 1, N, d).astype(np.float64)
    y, _, _ = lay.prefill(x)
    acc = np.zeros(d)
    for k in range(1, N + 1):
        zk = x[0, k - 1] + (alpha / k) * (Vm @ x[0, k - 1] + Vm @ acc)
        np.testing.assert_allclose(y[0, k - 1], zk, rtol=1e-12, atol=1e-13)
        acc += zk
    # scalar worked value: d = 1, alpha V = 1  =>  z_1 = 2 and z_k = k!/k! = 1 for k >= 2
    one = np.ones((1, 1))
    s = oracle.Layer({"Wq": 0 * one, "Wk": one, "Wv": one, "Wo": None, "W1": 0 * one, "W2": 0 * one}, 1,
                     norm_free=True, alpha=1.0)
    xs = np.zeros((1, 6, 1))
    xs[0, 0, 0] = 1.0
    ys, _, _ = s.prefill(xs)
    np.testing.assert_allclose(ys[0, :, 0], [2, 1, 1, 1, 1, 1], rtol=1e-13)


# ------------------------------------------------------------------------------------------
# P7  Schedule: the paper's worked examples and exact-once coverage (Appendix C).
# ------------------------------------------------------------------------------------------
def test_p7_schedule_examples_from_paper(oracle):
    ev = {e[0]: e for e in oracle.schedule(8)}
    with open(os.path.join(GOLDEN, "schedule_examples.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                row = tuple(int(v) for v in line.split())
                assert ev[row[0]] == row


@pytest.mark.parametrize("N", [1, 2, 3, 7, 8, 100, 257, 300])
def test_p7_schedule_covers_every_pair_once(oracle, N):
    ev = oracle.schedule(N)
    cover = np.zeros((N + 1, N + 1), dtype=np.int32)
    tiles_per_query = np.zeros(N + 1, dtype=np.int32)
    total = 0
    for (t, P, u, v, s, e) in ev:
        assert P & (P - 1) == 0 and t % P == 0 and (t // P) % 2 == 1
        assert (s, e) == (t - P + 1, t) and u == t + 1 and v == min(t + P, N) and u <= v
        cover[u:v + 1, s:e + 1] += 1
        tiles_per_query[u:v + 1] += 1
        total += P * (v - u + 1)
    for i in range(1, N + 1):
        assert (cover[i, 1:i] == 1).all() and (cover[i, i:] == 0).all()
        assert tiles_per_query[i] == bin(i - 1).count("1")
    assert total == N * (N - 1) // 2
    assert len(ev) == N - 1 if N > 1 else len(ev) == 0


# ------------------------------------------------------------------------------------------
# P8  The tiled algorithm (Algorithms 1 + 2, literal) equals the plain recurrence.
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N", [1, 2, 5, 16, 37, 64])
def test_p8_tiled_equals_naive(oracle, N):
    x, w, g = _small(41, B=2, N=N, d=24, H=3, F=40)
    lay = oracle.Layer(w, 3, gains=g, alpha=0.9, eps=1e-6, attn_scale=1.0)
    y, K, V = lay.prefill(x)
    y2, K2, V2 = lay.prefill_tiled(x)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(K2, K, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(V2, V, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("N,chunk", [(5, 4), (37, 4), (64, 16), (70, 16), (33, 32), (20, 32)])
def test_p8_chunked_schedule_equals_naive(oracle, N, chunk):
    """The schedule of a layer that knows its queries one chunk ahead (blocks of `chunk` keys and more replaced by one
    UpdateTile per chunk over all earlier keys) gives the plain recurrence's result: UpdateTile is exact for any
    partition of the keys (Appendix C)."""
    x, w, g = _small(43, B=2, N=N, d=24, H=3, F=40)
    lay = oracle.Layer(w, 3, gains=g, alpha=0.9, eps=1e-6, attn_scale=1.0)
    y, K, V = lay.prefill(x)
    y2, K2, V2 = lay.prefill_tiled(x, chunk=chunk)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(K2, K, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(V2, V, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------------------
# P9  Softmax special cases.
# ------------------------------------------------------------------------------------------
def test_p9_zero_queries_give_running_mean(oracle):
    x, w, g = _small(51, B=1, N=9)
    w = dict(w)
    w["Wq"] = np.zeros_like(w["Wq"])
    H, d = 2, 16
    eps = 1e-6                      # a zero query normalises to zero only with eps > 0
    lay = oracle.Layer(w, H, gains=g, eps=eps)
    y, K, V = lay.prefill(x)
    for i in range(9):
        vt = w["Wv"] @ _rms(x[0, i], g["g_attn"], eps)
        mean_v = (V[:i, 0].reshape(i, d).sum(axis=0) + vt) / (i + 1)
        hdd = x[0, i] + w["Wo"] @ mean_v
        z = hdd + w["W2"] @ _gelu(w["W1"] @ _rms(hdd, g["g_mlp"], eps))
        np.testing.assert_allclose(y[0, i], z, rtol=1e-12, atol=1e-13)


def test_p9_update_tile_any_split_any_order_equals_direct_softmax(oracle):
    nq, nkv, dh, scale = 5, 23, 8, 1.7
    q = gen.normal(52, 1, (nq, dh), 3.0).astype(np.float64)
    k = gen.normal(52, 2, (nkv, dh), 3.0).astype(np.float64)
    v = gen.normal(52, 3, (nkv, dh)).astype(np.float64)
    S = scale * q @ k.T
    Pm = np.exp(S - S.max(axis=1, keepdims=True))
    ref = (Pm / Pm.sum(axis=1, keepdims=True)) @ v
    for order in ([(0, 23)], [(0, 7), (7, 8), (8, 23)], [(16, 23), (0, 4), (4, 16)]):
        m = np.full(nq, -np.inf)
        l = np.zeros(nq)
        o = np.zeros((nq, dh))
        for (s, e) in order:
            oracle.update_tile(q, k[s:e], v[s:e], m, l, o, scale)
        np.testing.assert_allclose(o / l[:, None], ref, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(m, S.max(axis=1), rtol=1e-13, atol=0)
    # logits far beyond exp's range stay finite (max-subtraction), shifting all logits changes nothing
    m = np.full(nq, -np.inf); l = np.zeros(nq); o = np.zeros((nq, dh))
    oracle.update_tile(q * 40, k, v, m, l, o, scale)
    assert np.isfinite(o).all() and np.isfinite(l).all() and (l >= 1.0).all()


# ------------------------------------------------------------------------------------------
# P10  Independence of batch rows; relabelling heads.
# ------------------------------------------------------------------------------------------
def test_p10_batch_rows_independent_and_head_permutation(oracle):
    x, w, g = _small(61, B=3, N=10, d=24, H=3, F=40)
    lay = oracle.Layer(w, 3, gains=g)
    y, K, V = lay.prefill(x)
    y1, K1, V1 = lay.prefill(x[1:2])
    np.testing.assert_array_equal(y[1:2], y1)
    np.testing.assert_array_equal(K[:, 1:2], K1)
    dh = 8
    perm = np.concatenate([np.arange(2 * dh, 3 * dh), np.arange(0, dh), np.arange(dh, 2 * dh)])
    wp = dict(w)
    for n in ("Wq", "Wk", "Wv"):
        wp[n] = w[n][perm]
    wp["Wo"] = w["Wo"][:, perm]
    gp = dict(g)
    gp["g_q"], gp["g_k"] = g["g_q"][perm], g["g_k"][perm]
    yp, Kp, Vp = oracle.Layer(wp, 3, gains=gp).prefill(x)
    np.testing.assert_allclose(yp, y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Kp.reshape(10, 3, 24), K.reshape(10, 3, 24)[..., perm], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------------------------------
# P11  A prefill is a sequence of decode steps (Sec. 5, "one forward pass is essentially a
#      sequence of decode steps"; Sec. 7.3).
# ------------------------------------------------------------------------------------------
def test_p11_prefill_equals_prefill_then_decode(oracle):
    x, w, g = _small(71, B=2, N=13)
    lay = oracle.Layer(w, 2, gains=g, alpha=0.8)
    y, K, V = lay.prefill(x)
    n0 = 8
    y0, K0, V0 = lay.prefill(x[:, :n0], kv_cap=13)
    np.testing.assert_array_equal(y0, y[:, :n0])
    for t in range(n0, 13):
        yt = lay.decode_step(x[:, t], t, K0, V0)
        np.testing.assert_array_equal(yt, y[:, t])
    np.testing.assert_array_equal(K0, K)
    np.testing.assert_array_equal(V0, V)


# ------------------------------------------------------------------------------------------
# Threading modes give identical bits (batch-parallel, row-split and serial evaluation).
# ------------------------------------------------------------------------------------------
def test_thread_modes_bit_identical(oracle):
    li = gen.make_custom(81, "f32", 2, 6, 256, 4, 512)
    w = {k: v.astype(np.float64) for k, v in li.weights.items()}
    x = li.x.astype(np.float64)
    ref = oracle.Layer(w, 4, threads=1).prefill(x)
    for nt in (2, 4):
        got = oracle.Layer(w, 4, threads=nt).prefill(x)
        for a, b in zip(ref, got):
            np.testing.assert_array_equal(a, b)
    x8 = np.concatenate([x] * 4, axis=0)
    got8 = oracle.Layer(w, 4, threads=4).prefill(x8)
    np.testing.assert_array_equal(got8[0][:2], ref[0])
    # a single sequence: the matrix rows are split over the threads instead of the batch rows
    got1 = oracle.Layer(w, 4, threads=4).prefill(x[:1])
    np.testing.assert_array_equal(got1[0], ref[0][:1])
    np.testing.assert_array_equal(got1[1], ref[1][:, :1])


# ------------------------------------------------------------------------------------------
# Stack helpers: embedding lookup, final norm + read-out, layers fed one into the next (Sec. 2).
# ------------------------------------------------------------------------------------------
def test_stack_embed_is_row_lookup(oracle):
    rng = np.random.default_rng(5)
    table = rng.standard_normal((11, 6))
    ids = np.array([[3, 0, 10, 3], [7, 7, 1, 2]])
    x = oracle.embed(table, ids)
    assert x.shape == (2, 4, 6)
    for b in range(2):
        for n in range(4):
            assert list(x[b, n]) == list(table[ids[b, n]])


def test_stack_lm_head_closed_forms(oracle):
    rng = np.random.default_rng(6)
    d, vocab = 8, 5
    W = rng.standard_normal((vocab, d))
    signs = np.array([1, -1, 1, 1, -1, -1, 1, -1], dtype=np.float64)
    # a vector of constant magnitude normalises to its sign pattern (eps = 0): logits are signed row sums
    want = [sum(W[v, k] * signs[k] for k in range(d)) for v in range(vocab)]
    got = oracle.lm_head(W, (3.7 * signs)[None, :], eps=0.0)
    np.testing.assert_allclose(got[0], want, rtol=1e-14)
    # scale invariance at eps = 0, and a gain equals a column scaling of the matrix
    z = rng.standard_normal((3, d))
    np.testing.assert_allclose(oracle.lm_head(W, 5.0 * z, eps=0.0), oracle.lm_head(W, z, eps=0.0), rtol=1e-13)
    g = rng.uniform(0.5, 1.5, d)
    np.testing.assert_allclose(oracle.lm_head(W, z, g_final=g, eps=1e-6), oracle.lm_head(W * g[None, :], z, eps=1e-6),
                               rtol=1e-13)
    # eps enters under the root next to the mean square
    z1 = np.full((1, d), 2.0)
    np.testing.assert_allclose(oracle.lm_head(W, z1, eps=5.0)[0], W.sum(axis=1) * 2.0 / 3.0, rtol=1e-14)
    # norm-free: plain projection
    np.testing.assert_allclose(oracle.lm_head(W, z, norm_free=True), np.einsum("vk,bk->bv", W, z), rtol=1e-13)


def test_stack_composes_layers_and_decodes(oracle):
    rng = np.random.default_rng(7)
    d, H, F, vocab, B, N = 16, 2, 32, 19, 2, 11
    table = rng.standard_normal((vocab, d)) * 0.5
    W_lm = rng.standard_normal((vocab, d))
    ids = rng.integers(0, vocab, size=(B, N))
    lays = []
    for l in range(3):
        li = gen.make_custom(90 + l, "f32", 1, 1, d, H, F, w_std=0.3, gains="random")
        lays.append(oracle.Layer({k: v.astype(np.float64) for k, v in li.weights.items()}, H,
                                 gains={k: v.astype(np.float64) for k, v in li.gains.items()}, alpha=1 / math.sqrt(3)))
    st = oracle.Stack(lays, table, W_lm)
    out, logits = st.prefill(ids, N, kv_cap=N)
    # layer l+1 reads layer l's output; layer 0 reads the looked-up rows
    x = table[ids]
    for l in range(3):
        y, K, V = lays[l].prefill(x)
        np.testing.assert_array_equal(out[l][0], y)
        np.testing.assert_array_equal(out[l][1], K)
        x = y
    np.testing.assert_allclose(logits, _rms(x[:, -1], eps=1e-6) @ W_lm.T, rtol=1e-12)
    # a shorter prefill followed by decoding steps reproduces the longer prefill (Sec. 7.3), layer by layer
    st2 = oracle.Stack(lays, table, W_lm)
    n0 = 6
    out0, _ = st2.prefill(ids, n0, kv_cap=N)
    for t in range(n0, N):
        ys, lg = st2.decode_step(ids, t)
        for l in range(3):
            np.testing.assert_array_equal(ys[l], out[l][0][:, t])
    np.testing.assert_allclose(lg, logits, rtol=1e-12)
    for l in range(3):
        np.testing.assert_array_equal(st2.K[l], out[l][1])


# ------------------------------------------------------------------------------------------
# P12  ALiBi (Appendix D: the trained models use ALiBi positional biases with maximum bias 8.0; Press et al.:
#      logit(i, j) -= m_h (i - j), head slopes a geometric sequence m_h = 2^(-8 (h+1) / H)).
# ------------------------------------------------------------------------------------------
def test_p12_alibi_zero_queries_give_geometric_weights(oracle):
    """Wq = 0: every content logit vanishes, so position t (0-based) spreads its attention over keys 0..t-1 and its own
    temporary pair as r^(t-j) / sum_{i=0..t} r^i with r = exp(-m_h): checks the slopes head by head, the sign, and that
    the temporary pair sits at distance 0 and the newest persistent key at distance 1."""
    H, N, beta = 4, 9, 8.0
    x, w, g = _small(61, B=1, N=N, d=32, H=H, F=16)
    w = dict(w)
    w["Wq"] = np.zeros_like(w["Wq"])
    _, _, _, attw = oracle.Layer(w, H, gains=g, alibi_max_bias=beta).prefill(x, want_attw=True)
    for h in range(H):
        r = math.exp(-(2.0 ** (-beta * (h + 1) / H)))
        for t in range(N):
            ref = np.array([r ** (t - j) for j in range(t + 1)])
            np.testing.assert_allclose(attw[0, h, t, :t + 1], ref / ref.sum(), rtol=1e-12, atol=1e-15)
    # H = 8, beta = 8: the slopes of Press et al., 1/2, 1/4, ..., 1/256
    H = 8
    x, w, g = _small(62, B=1, N=3, d=32, H=H, F=16)
    w = dict(w)
    w["Wq"] = np.zeros_like(w["Wq"])
    _, _, _, attw = oracle.Layer(w, H, gains=g, alibi_max_bias=8.0).prefill(x, want_attw=True)
    for h in range(H):
        m = 0.5 ** (h + 1)
        np.testing.assert_allclose(attw[0, h, 1, 0] / attw[0, h, 1, 1], math.exp(-m), rtol=1e-12)


@pytest.mark.parametrize("beta", [8.0, 3.0])
def test_p12_alibi_dense_restatement_and_fixed_point(oracle, beta):
    x, w, g = _small(63, B=2, N=14, d=24, H=3, F=40)
    alpha, eps, scale = 0.7, 1e-6, 0.5
    lay = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale, alibi_max_bias=beta)
    y, K, V = lay.prefill(x)
    y0, _, _ = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale).prefill(x)
    assert np.abs(y - y0).max() > 1e-3                      # the bias matters at this size
    for b in range(2):
        np.testing.assert_allclose(y[b], _rt_numpy(x[b], w, g, 3, alpha=alpha, eps=eps, scale=scale, alibi=beta),
                                   rtol=1e-11, atol=1e-12)
        z2, Kp, Vp = _parallel_recompute(x[b], y[b], w, g, 3, alpha, eps, scale, alibi=beta)
        np.testing.assert_allclose(z2, y[b], rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(K[:, b], Kp, rtol=1e-10, atol=1e-11)
    # a bias of the wrong sign is not a fixed point
    bad, _, _ = _parallel_recompute(x[0], y[0], w, g, 3, alpha, eps, scale, alibi=-beta)
    assert np.abs(bad - y[0]).max() > 1e-3
    # the tiled algorithm (Appendix C) with the bias carried into every tile, and its chunked variant; decoding
    for chunk in (0, 4):
        y2, K2, _ = lay.prefill_tiled(x, chunk=chunk)
        np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(K2, K, rtol=1e-12, atol=1e-12)
    yp, Kp2, Vp2 = lay.prefill(x[:, :9], kv_cap=14)
    for t in range(9, 14):
        yt = lay.decode_step(x[:, t], t, Kp2, Vp2)
        np.testing.assert_array_equal(yt, y[:, t])
    # beta = 0 is the layer without positions, bit for bit
    y3, _, _ = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale, alibi_max_bias=0.0).prefill(x)
    np.testing.assert_array_equal(y3, y0)


# ------------------------------------------------------------------------------------------
# P13  Blocked recurrence (Sec. 8: "recurrence executed over blocks of steps"; reading: persistent pairs across blocks,
#      temporary pairs inside a block).
# ------------------------------------------------------------------------------------------
def _blocked_fixed_point(x, z, w, g, H, S, alpha, eps, scale, alibi=0.0):
    """Dense restatement for one sequence: with z given, key j of query i is the persistent pair (from z_j) when j lies
    in an earlier block and the temporary pair (from x_j) when it lies in i's own block, j <= i."""
    N, d = x.shape
    dh = d // H
    gq, gk = g["g_q"].reshape(H, dh), g["g_k"].reshape(H, dh)
    n = _rms(x, g["g_attn"], eps)
    Q = _rms((n @ w["Wq"].T).reshape(N, H, dh), gq, eps)
    Kt = _rms((n @ w["Wk"].T).reshape(N, H, dh), gk, eps)
    Vt = (n @ w["Wv"].T).reshape(N, H, dh)
    r = _rms(z, g["g_kv"], eps)
    Kp = _rms((r @ w["Wk"].T).reshape(N, H, dh), gk, eps)
    Vp = (r @ w["Wv"].T).reshape(N, H, dh)
    i, j = np.arange(N)[:, None], np.arange(N)[None, :]
    same = (i // S) == (j // S)
    cat = np.zeros((N, H, dh))
    for h in range(H):
        Sm = scale * np.where(same, Q[:, h] @ Kt[:, h].T, Q[:, h] @ Kp[:, h].T)
        if alibi:
            Sm = Sm - 2.0 ** (-alibi * (h + 1) / H) * (i - j)
        Sm = np.where(j <= i, Sm, -np.inf)
        P = np.exp(Sm - Sm.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        cat[:, h] = (P * same) @ Vt[:, h] + (P * ~same) @ Vp[:, h]
    a = cat.reshape(N, d) @ w["Wo"].T
    hdd = x + alpha * a
    return hdd + alpha * (_gelu(_rms(hdd, g["g_mlp"], eps) @ w["W1"].T) @ w["W2"].T), Kp, Vp


@pytest.mark.parametrize("S,beta", [(4, 0.0), (8, 8.0), (5, 0.0)])
def test_p13_blocked_recurrence(oracle, S, beta):
    x, w, g = _small(71, B=2, N=22, d=24, H=3, F=40)
    alpha, eps, scale = 0.6, 1e-5, 0.5
    lay = oracle.Layer(w, 3, gains=g, alpha=alpha, eps=eps, attn_scale=scale, alibi_max_bias=beta)
    y, K, V = lay.prefill_blocked(x, S)
    # the two ends of the family: one position per block is the RT layer, one block is the Transformer layer
    y1, K1, V1 = lay.prefill_blocked(x, 1)
    yr, Kr, Vr = lay.prefill(x)
    np.testing.assert_array_equal(y1, yr)
    np.testing.assert_array_equal(K1, Kr)
    yN, KN, VN = lay.prefill_blocked(x, 64)
    yT, KT, VT = lay.transformer(x)
    np.testing.assert_allclose(yN, yT, rtol=1e-12, atol=1e-13)
    # in between it is neither ...
    assert np.abs(y - yr).max() > 1e-3 and np.abs(y - yT).max() > 1e-3
    # ... but the fixed point of the dense restatement with the block mask, with persistent pairs projected from its output
    for b in range(2):
        z2, Kp, Vp = _blocked_fixed_point(x[b], y[b], w, g, 3, S, alpha, eps, scale, alibi=beta)
        np.testing.assert_allclose(z2, y[b], rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(K[:, b], Kp, rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(V[:, b], Vp, rtol=1e-10, atol=1e-11)
    # the first block sees no persistent pair at all: it is the Transformer layer on those positions
    np.testing.assert_allclose(y[:, :S], yT[:, :S], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------------------------------
# Conditioning of the exact map on the stack workload's first-layer input (a property of the definition of
# Sec. 2.2, measured on the oracle alone).  With embedding entries ~ N(0, 0.02^2) fed to the layer as they are and the
# paper's unscaled logits, z = x + branch is dominated by the branch, every persistent key is a normalised copy of
# it, the softmax over logits of standard deviation 8 is sharp, and a relative input perturbation of one bf16
# rounding (2^-9) comes out amplified far beyond the 2e-2 the GPU path is held to - so no finite-precision
# evaluation can be compared with the oracle at a tolerance there.  The same table with logits scaled by 1/8, and
# the table multiplied by 50 (entries ~ N(0, 1), like x in the single-layer workloads), are benign.  The GPU parity
# tests of the stack run on the two benign variants for this reason.
# ------------------------------------------------------------------------------------------
def test_stack_workload_conditioning_literal_table_vs_benign_variants(oracle):
    wl = gen.WORKLOADS["cfg5"]
    B, N = 2, 64
    ids = gen.make_token_ids(wl)[:B, :N]
    table = gen.make_embedding_tables(wl)["embedding"].astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in gen.make_layer_weights(wl.seed, 0, wl.d, wl.F, wl.dtype).items()}
    rel = 2.0 ** -9
    noise = 1.0 + np.random.default_rng(11).uniform(-rel, rel, (B, N, wl.d))

    def amplification(mult, attn_scale):
        lay = oracle.Layer(w, wl.H, alpha=wl.resid_scale, eps=1e-6, attn_scale=attn_scale)
        x = oracle.embed(table * mult, ids)
        y0, y1 = lay.prefill(x)[0], lay.prefill(x * noise)[0]
        err = np.linalg.norm(y1 - y0, axis=-1) / np.linalg.norm(y0, axis=-1)
        return err.max(axis=0) / rel          # curve over the position

    literal = amplification(1.0, 1.0)
    assert literal[0] < 3.0                    # a single position: one softmax weight, nothing to amplify
    assert literal[32:].max() > 10.0, literal[32:].max()
    assert amplification(50.0, 1.0).max() < 3.0
    assert amplification(1.0, 0.125).max() < 3.0
