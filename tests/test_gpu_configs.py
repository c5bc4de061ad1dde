"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times
(default engine selection, default p_min), element by element against the CPU oracle."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, BRANCH_TOL, error_curves, summarize, oracle_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _full(oracle, name, N=None, engine="persistent"):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    wl = gen.WORKLOADS[name]
    N = N or wl.N
    li = gen.make_layer_inputs(wl, N=N)
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, wl.H, alpha=wl.resid_scale, eps=1e-6).prefill(x64)
    ctx = binding.RTContext(wl.d, wl.H, wl.F, wl.B, N, wl.dtype, resid_scale=wl.resid_scale, rms_eps=1e-6,
                            stream=torch.cuda.current_stream().cuda_stream)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, wl.dtype)
        y, K, V = tio.prefill(ctx, dl, tio.to_device(li.x, wl.dtype))
        torch.cuda.synchronize()
        assert ctx.device_wait_expired() == 0
        assert ctx.engine_name() == engine
        got = (tio.to_host(y), tio.to_host(K), tio.to_host(V))
    finally:
        ctx.rt_destroy()
    cur = error_curves(x64, ref, got)
    print("\n  [%s N=%d %s] %s" % (name, N, engine, summarize(cur)))
    for k in ("y", "K", "V"):
        assert cur[k].max() <= TOL[wl.dtype], "%s error %.3e at position %d" % (k, cur[k].max(), int(np.argmax(cur[k])))
    assert cur["branch"].max() <= BRANCH_TOL[wl.dtype], "branch error %.3e at position %d" % (
        cur["branch"].max(), int(np.argmax(cur["branch"])))
    return cur


def test_config1_fp32_full(oracle):
    cur = _full(oracle, "cfg1", engine="stepwise")
    assert cur["branch"].max() < 1e-4


def test_config2_bf16_full(oracle):
    _full(oracle, "cfg2")


def test_config3_bf16_full_headline(oracle):
    _full(oracle, "cfg3")


@pytest.mark.parametrize("N", [1024, 2048])
def test_config4_sweep_prefixes(oracle, N):
    _full(oracle, "cfg4_8192", N=N)


@pytest.mark.parametrize("N", [4096, 8192])
def test_config4_long_sequences(N):
    """N = 4096 and 8192 (B = 2), where Algorithm 1's blocks of 2048 and 4096 keys and the upper partial-state slots
    first come into play.  (1) Against the fp64 oracle: 34 positions of its run at N = 8192 are stored by
    oracle/write_golden.py (first and last positions, both sides of the 1024 / 2048 / 4096 / 6144 block boundaries,
    scattered ones); the layer is causal and the shorter input a prefix of the longer, so the rows below 4096 are
    the N = 4096 run's references too.  y, K, V at each stored position within the tolerance.  (2) Properties that
    hold at any length: the first 2048 positions agree with the run of length 2048 (which the oracle checks element
    by element), and sampled late positions re-evaluated by rt_decode_step - plain attention over the whole cache,
    no tiling, no stored partial states, different kernels - agree within twice the tolerance."""
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    import os
    from paper_2604_21215_amd import binding, torch_io as tio
    from tests.parity_util import rel_err_rows
    wl = gen.WORKLOADS["cfg4_8192"]
    li = gen.make_layer_inputs(wl, N=N)
    g = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_rows_sweep_b2_n8192.npz"))
    full = gen.make_layer_inputs(wl).x.astype(np.float64) if N == wl.N else None
    if full is not None:   # the stored rows belong to exactly these inputs
        fp = np.array([full.sum(), np.abs(full).sum(), li.weights["W2"].astype(np.float64).sum()])
        np.testing.assert_allclose(g["fingerprint"], fp, rtol=1e-12)
    ctx = binding.RTContext(wl.d, wl.H, wl.F, wl.B, N, wl.dtype, rms_eps=1e-6, stream=torch.cuda.current_stream().cuda_stream)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, wl.dtype)
        xd = tio.to_device(li.x, wl.dtype)
        y, K, V = tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        assert ctx.device_wait_expired() == 0 and ctx.engine_name() == "persistent"
        pos = g["positions_y"]
        sel = pos < N
        idx = pos[sel].tolist()
        ey = rel_err_rows(tio.to_host(y[:, idx]).transpose(1, 0, 2), g["y"][0][sel].astype(np.float64)).max(axis=1)
        eK = rel_err_rows(tio.to_host(K[idx]), g["K"][0][sel].astype(np.float64)).reshape(len(idx), -1).max(axis=1)
        eV = rel_err_rows(tio.to_host(V[idx]), g["V"][0][sel].astype(np.float64)).reshape(len(idx), -1).max(axis=1)
        xs = li.x.astype(np.float64)[:, idx].transpose(1, 0, 2)
        ebr = rel_err_rows(tio.to_host(y[:, idx]).transpose(1, 0, 2) - xs, g["y"][0][sel].astype(np.float64) - xs).max(axis=1)
        print("\n  [cfg4 N=%d vs oracle rows] y %.1e K %.1e V %.1e branch %.1e over positions %s" %
              (N, ey.max(), eK.max(), eV.max(), ebr.max(), idx))
        print("    per position: " + " ".join("%d:%.1e/%.1e/%.1e" % (p, a, b, c) for p, a, b, c in zip(idx, ey, eK, eV)))
        assert max(ey.max(), eK.max(), eV.max()) <= TOL[wl.dtype]
        assert ebr.max() <= BRANCH_TOL[wl.dtype]
        ys, Ks, Vs = tio.prefill(ctx, dl, xd[:, :2048].contiguous())
        torch.cuda.synchronize()
        pre = [rel_err_rows(tio.to_host(ys), tio.to_host(y[:, :2048])).max(),
               rel_err_rows(tio.to_host(Ks), tio.to_host(K[:2048])).max(),
               rel_err_rows(tio.to_host(Vs), tio.to_host(V[:2048])).max()]
        print("  [cfg4 N=%d: first 2048 positions vs the run of length 2048] y %.1e K %.1e V %.1e" % (N, *pre))
        assert max(pre) <= 0.5 * TOL[wl.dtype]
        worst = np.zeros(3)
        for t in (N - 1, N - 2, N // 2, N // 2 + 1, 3 * N // 4 - 1, N // 2 + N // 8 + 37, 2048 + 33):
            Kc, Vc = K.clone(), V.clone()
            y_t = torch.empty((wl.B, wl.d), dtype=y.dtype, device=y.device)
            ctx.rt_decode_step(dl.struct, xd[:, t].contiguous(), t, y_t, Kc, Vc)
            torch.cuda.synchronize()
            e = [rel_err_rows(tio.to_host(y_t), tio.to_host(y[:, t])).max(),
                 rel_err_rows(tio.to_host(Kc[t]), tio.to_host(K[t])).max(),
                 rel_err_rows(tio.to_host(Vc[t]), tio.to_host(V[t])).max()]
            worst = np.maximum(worst, e)
        print("  [cfg4 N=%d: decode re-evaluation of 7 late positions vs prefill] y %.1e K %.1e V %.1e" % (N, *worst))
        assert worst.max() <= 2 * TOL[wl.dtype]
    finally:
        ctx.rt_destroy()


def test_config3_loop_free_layers_full_size(oracle):
    """The loop-free layers at the headline size (B = 8, N = 2048, d = 1024: 16384 rows through the LDS-tiled products, 128
    (b, h) x 16 query tiles through the masked attention pass), as bench.py times them.  All three layers are causal, so
    the first Np positions depend on the first Np inputs only and the oracle is run on that prefix; beyond it the
    recompute is checked through its defining property: fed with the output of rt_layer_prefill it reproduces that output
    and its K, V at every position."""
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    wl = gen.WORKLOADS["cfg3"]
    li = gen.make_layer_inputs(wl)
    Np = 256
    x64p = li.x[:, :Np].astype(np.float64)
    lay = oracle_layer(oracle, li, wl.H, alpha=wl.resid_scale, eps=1e-6)
    ctx = binding.RTContext(wl.d, wl.H, wl.F, wl.B, wl.N, wl.dtype, resid_scale=wl.resid_scale, rms_eps=1e-6,
                            stream=torch.cuda.current_stream().cuda_stream)
    tol = TOL[wl.dtype]

    def check(name, xs, ref, got):
        cur = error_curves(xs, ref, got)
        print("\n  [cfg3 full size, %s] %s" % (name, summarize(cur)))
        for k in ("y", "K", "V"):
            assert cur[k].max() <= tol, "%s %s: %.3e at position %d" % (name, k, cur[k].max(), int(np.argmax(cur[k])))

    try:
        dl = tio.DeviceLayer(li.weights, li.gains, wl.dtype)
        xd = tio.to_device(li.x, wl.dtype)
        y = torch.empty_like(xd)
        K = torch.zeros((wl.N, wl.B, wl.H, wl.d // wl.H), dtype=xd.dtype, device=xd.device)
        V = torch.zeros_like(K)
        prefix = lambda: (tio.to_host(y)[:, :Np], tio.to_host(K)[:Np], tio.to_host(V)[:Np])

        ctx.rt_transformer_layer(dl.struct, xd, y, K, V)
        torch.cuda.synchronize()
        check("Transformer layer, first %d positions vs oracle" % Np, x64p, lay.transformer(x64p), prefix())

        ctx.rt_layer_prefill_blocked(dl.struct, xd, 32, y, K, V)
        torch.cuda.synchronize()
        check("blocked recurrence (32), first %d positions vs oracle" % Np, x64p, lay.prefill_blocked(x64p, 32), prefix())

        y1, K1, V1 = tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "persistent"
        ctx.rt_layer_recompute(dl.struct, xd, y1, y, K, V)
        torch.cuda.synchronize()
        check("recompute of the prefill's output, first %d positions vs oracle" % Np, x64p, lay.prefill(x64p), prefix())
        check("recompute of the prefill's output vs that output, all positions", li.x.astype(np.float64),
              (tio.to_host(y1), tio.to_host(K1), tio.to_host(V1)), (tio.to_host(y), tio.to_host(K), tio.to_host(V)))
    finally:
        ctx.rt_destroy()
