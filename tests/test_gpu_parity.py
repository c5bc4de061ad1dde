"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element on the same
seeded buffers, reported as error curves over position.

Tolerance (norm-wise relative error per position, max over batch rows / heads):
    fp32 storage 1e-4, bf16 storage 2e-2  -- for y, K and V separately.
"""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, error_curves, summarize, oracle_layer

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    from paper_2604_21215_amd import binding, torch_io
    return binding, torch_io


def _run_case(oracle, dtype, B, N, d, H, F, *, flags=0, p_min=0, gains="unit", seed=5, alpha=1.0, scale=1.0,
              eps=1e-6, kv_cap=None, li=None, tol_scale=1.0, expect_engine=None, alibi=0.0, n_decode=0):
    binding, tio = _gpu()
    if li is None:
        li = gen.make_custom(seed, dtype, B, N, d, H, F, gains=gains)
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, H, alpha=alpha, attn_scale=scale, eps=eps, alibi_max_bias=alibi).prefill(x64)
    ctx = binding.RTContext(d, H, F, B, N, dtype, p_min=p_min, resid_scale=alpha, attn_scale=scale, rms_eps=eps,
                            flags=flags, alibi_max_bias=alibi)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, dtype)
        xd = tio.to_device(li.x, dtype)
        y, K, V = tio.prefill(ctx, dl, xd, kv_cap=kv_cap)
        torch.cuda.synchronize()
        assert ctx.device_wait_expired() == 0
        if expect_engine:
            assert ctx.engine_name() == expect_engine
        got = (tio.to_host(y), tio.to_host(K), tio.to_host(V))
        # the last n_decode positions once more, one rt_decode_step each over the cache the prefill left
        for t in range(N - n_decode, N):
            y_t = torch.empty_like(xd[:, t])
            ctx.rt_decode_step(dl.struct, xd[:, t].contiguous(), t, y_t, K, V)
            torch.cuda.synchronize()
            e = np.linalg.norm(tio.to_host(y_t) - ref[0][:, t], axis=-1) / np.linalg.norm(ref[0][:, t], axis=-1)
            assert e.max() <= TOL[dtype] * tol_scale, "decode step %d: %.3e" % (t, e.max())
    finally:
        ctx.rt_destroy()
    cur = error_curves(x64, ref, got)
    print("\n  [%s B=%d N=%d d=%d p_min=%d flags=%#x] %s" % (dtype, B, N, d, p_min, flags, summarize(cur)))
    tol = TOL[dtype] * tol_scale
    for name in ("y", "K", "V"):
        t_bad = int(np.argmax(cur[name]))
        assert cur[name].max() <= tol, "%s: error %.3e at position %d exceeds %.1e" % (name, cur[name].max(), t_bad, tol)
    if kv_cap is not None and kv_cap > N:
        assert np.all(got[1][N:] == 0) and np.all(got[2][N:] == 0)      # rows beyond N untouched
    return cur


def _flags():
    from paper_2604_21215_amd import binding
    return binding


# ----------------------------------------------------------------------------- per-position engine
@pytest.mark.parametrize("N", [1, 2, 3, 7, 33, 100])
def test_stepwise_f32_small_and_ragged_lengths(oracle, N):
    b = _flags()
    _run_case(oracle, "f32", 2, N, 128, 2, 512, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=4, expect_engine="stepwise")


@pytest.mark.parametrize("p_min", [1, 2, 8, 32, 256])
def test_stepwise_f32_threshold_does_not_change_results(oracle, p_min):
    b = _flags()
    _run_case(oracle, "f32", 1, 150, 128, 2, 256, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=p_min)


def test_stepwise_f32_gains_scales_and_batch_tiles(oracle):
    b = _flags()
    _run_case(oracle, "f32", 11, 70, 128, 2, 264, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=8, gains="random", alpha=0.7,
              scale=0.5, kv_cap=80)
    _run_case(oracle, "f32", 3, 40, 192, 3, 512, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=4, gains="random",
              alpha=1.0 / np.sqrt(12.0), scale=0.125, eps=0.0)


def test_stepwise_config1_f32(oracle):
    """Configuration 1: fp32, B=1, N=256, d=128, 2 heads, hidden 512."""
    b = _flags()
    wl = gen.WORKLOADS["cfg1"]
    li = gen.make_layer_inputs(wl)
    cur = _run_case(oracle, "f32", wl.B, wl.N, wl.d, wl.H, wl.F, flags=b.RT_FLAG_ENGINE_STEPWISE, li=li)
    assert cur["branch"].max() < 1e-4


def test_stepwise_bf16_plain_alu_and_mfma_agree_with_oracle(oracle):
    b = _flags()
    _run_case(oracle, "bf16", 2, 200, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE | b.RT_FLAG_NO_MFMA, p_min=8)
    _run_case(oracle, "bf16", 2, 200, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=32)
    _run_case(oracle, "bf16", 3, 300, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=32, gains="random",
              alpha=0.7, scale=0.5, kv_cap=320)
    _run_case(oracle, "bf16", 5, 333, 320, 5, 1280, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=64)   # odd head count, ragged N


# ----------------------------------------------------------------------------- ALiBi
@pytest.mark.parametrize("N,p_min", [(100, 4), (150, 32), (40, 1)])
def test_alibi_stepwise_f32(oracle, N, p_min):
    """Linear positional bias (maximum bias 8, slopes 2^(-8 (h+1)/H)) through every plain-ALU kernel: direct window,
    stored partial states of several levels, the temporary pair at distance 0, and decoding steps over the cache."""
    b = _flags()
    _run_case(oracle, "f32", 2, N, 256, 4, 512, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=p_min, alibi=8.0, gains="random",
              scale=0.5, n_decode=3, expect_engine="stepwise")


def test_alibi_bf16_mfma_tiles(oracle):
    """The matrix-core tiles of the per-position engine with the bias: 32-key blocks (wave kernel), 64 .. 256-key
    blocks (LDS-staged kernel, several chunks per block), a ragged tail."""
    b = _flags()
    _run_case(oracle, "bf16", 2, 600, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=32, alibi=8.0, n_decode=2,
              expect_engine="stepwise")
    _run_case(oracle, "bf16", 3, 333, 320, 5, 1280, p_min=64, alibi=3.0, scale=0.5, gains="random", expect_engine="stepwise")
    _run_case(oracle, "bf16", 2, 200, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE | b.RT_FLAG_NO_MFMA, p_min=8, alibi=8.0)


def test_alibi_persistent_engine(oracle):
    """The single-launch engine with the bias: LDS window (newest key at distance 1), stored partial states from the
    in-workgroup tiles (32 .. 128 keys) and from the grid-wide tiles (256 and 512 keys), several heads per workgroup
    slot, gains and a logit scale."""
    _run_case(oracle, "bf16", 2, 600, 256, 4, 1024, alibi=8.0, n_decode=2, expect_engine="persistent")
    _run_case(oracle, "bf16", 3, 700, 1024, 16, 4096, alibi=8.0, expect_engine="persistent")
    _run_case(oracle, "bf16", 8, 300, 512, 8, 2048, alibi=3.0, scale=0.5, gains="random", alpha=0.7, expect_engine="persistent")


def test_alibi_rejects_a_negative_bias():
    binding, _ = _gpu()
    with pytest.raises(binding.RTError):
        binding.RTContext(256, 4, 1024, 2, 64, "bf16", alibi_max_bias=-1.0)


def test_cross_block_tiles_with_several_query_blocks(oracle):
    """Blocks of 256 and 512 keys: the LDS-staged tile kernel runs with two and more 128-query workgroups per
    (b, h), a ragged last workgroup (N = 700: the 512-key block serves 188 queries) and 16 x 3 = 48 (b, h)
    problems dealt over the 8 XCD slots."""
    b = _flags()
    _run_case(oracle, "bf16", 3, 700, 1024, 16, 4096, flags=b.RT_FLAG_ENGINE_STEPWISE, p_min=64, expect_engine="stepwise")


def test_cross_block_event_rerun_and_argument_checks(oracle):
    """rt_cross_block_event re-runs one tile on the state of the last prefill; the prefill's outputs stay as
    they were and a following prefill gives the same bits as before."""
    binding, tio = _gpu()
    B, N, d, H, F = 2, 300, 256, 4, 1024
    li = gen.make_custom(9, "bf16", B, N, d, H, F)
    for flags in (binding.RT_FLAG_ENGINE_STEPWISE, binding.RT_FLAG_ENGINE_PERSISTENT):
        ctx = binding.RTContext(d, H, F, B, N, "bf16", p_min=32, flags=flags)
        try:
            dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
            xd = tio.to_device(li.x, "bf16")
            K0 = torch.zeros((N, B, H, 64), dtype=torch.bfloat16, device="cuda:0")
            with pytest.raises(binding.RTError):
                ctx.rt_cross_block_event(K0, K0, 128, 128, 128)          # nothing has run yet
            y, K, V = tio.prefill(ctx, dl, xd)
            torch.cuda.synchronize()
            y0 = y.clone()
            for t1, P, nq in ((128, 128, 128), (256, 256, 44), (64, 64, 64), (32, 32, 32)):
                ctx.rt_cross_block_event(K, V, t1, P, nq)
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), y0.view(torch.int16))
            for bad in ((128, 128, 129), (100, 128, 10), (128, 96, 10), (256, 256, 45), (0, 128, 1), (128, 16, 16)):
                with pytest.raises(binding.RTError):
                    ctx.rt_cross_block_event(K, V, *bad)
            y2, _, _ = tio.prefill(ctx, dl, xd)
            torch.cuda.synchronize()
            assert torch.equal(y2.view(torch.int16), y0.view(torch.int16))
        finally:
            ctx.rt_destroy()


def test_stepwise_hip_graph_replay_matches(oracle):
    b = _flags()
    _run_case(oracle, "bf16", 2, 130, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_STEPWISE | b.RT_FLAG_HIP_GRAPH, p_min=32,
              expect_engine="stepwise+graph")


# ----------------------------------------------------------------------------- persistent engine
@pytest.mark.parametrize("B,N", [(1, 1), (2, 2), (2, 5), (3, 33), (2, 34), (5, 97), (16, 130)])
def test_persistent_small_and_ragged(oracle, B, N):
    b = _flags()
    _run_case(oracle, "bf16", B, N, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_PERSISTENT, expect_engine="persistent")


def test_persistent_full_batch_at_the_headline_width(oracle):
    """B = 16, d = 1024: every one of the 256 workgroups owns a (b, h) (merging and helper wavefront in each), 16 batch rows
    fill the matrix instructions' column dimension and the staged activations take their largest LDS share."""
    b = _flags()
    _run_case(oracle, "bf16", 16, 100, 1024, 16, 4096, flags=b.RT_FLAG_ENGINE_PERSISTENT, expect_engine="persistent")


@pytest.mark.parametrize("B,N,d", [(35, 70, 256), (20, 40, 1024)])
def test_persistent_batches_beyond_its_rows_run_in_chunks(oracle, B, N, d):
    """More sequences than the single-launch engine stages at once (16): the call runs chunks of 16 rows one after the
    other (16 + 16 + 3; 16 + 4) and copies each chunk's pairs into the position-major cache; cache rows beyond N stay
    untouched and a decoding step over the assembled cache agrees with the oracle."""
    _run_case(oracle, "bf16", B, N, d, d // 64, 4 * d, gains="random", scale=0.5, alpha=0.7, kv_cap=N + 5, n_decode=1,
              expect_engine="persistent")


def test_many_sequences_take_the_engines_cut_for_them(oracle):
    """rt_layer_prefill by batch size: up to 48 sequences chunks of 16 rows on the single-launch engine, from 49 to 128 the
    layer-wavefront engine with one layer, beyond that one position of all sequences per step with batched matrix products
    (each the fastest there): same results, same bounds."""
    _run_case(oracle, "bf16", 60, 70, 256, 4, 1024, gains="random", scale=0.5, alpha=0.7, kv_cap=72, n_decode=1,
              expect_engine="wavefront")
    _run_case(oracle, "bf16", 130, 70, 256, 4, 1024, gains="random", scale=0.5, alpha=0.7, kv_cap=72, n_decode=1,
              expect_engine="position-batched")
    # the largest batch a context takes: 1024 rows per step (other tile shapes of the products than at 130)
    _run_case(oracle, "bf16", 1024, 34, 256, 4, 1024, gains="random", scale=0.5, alpha=0.7, n_decode=1,
              expect_engine="position-batched")


def test_persistent_gains_scales_levels(oracle):
    b = _flags()
    _run_case(oracle, "bf16", 3, 300, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_PERSISTENT, gains="random", alpha=0.7,
              scale=0.5, kv_cap=310, expect_engine="persistent")
    _run_case(oracle, "bf16", 2, 200, 512, 8, 2048, flags=b.RT_FLAG_ENGINE_PERSISTENT, p_min=64, expect_engine="persistent")
    _run_case(oracle, "bf16", 2, 300, 256, 4, 1024, flags=b.RT_FLAG_ENGINE_PERSISTENT, p_min=128,
              expect_engine="persistent")                       # window re-read from K, V instead of LDS


def test_persistent_is_the_default_engine_and_repeats_bit_identically(oracle):
    binding, tio = _gpu()
    li = gen.make_custom(4, "bf16", 4, 161, 768, 12, 3072)
    ctx = binding.RTContext(768, 12, 3072, 4, 200, "bf16")
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
        xd = tio.to_device(li.x, "bf16")
        a = tio.prefill(ctx, dl, xd)
        b2 = tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "persistent" and ctx.device_wait_expired() == 0
        for u, v in zip(a, b2):
            assert torch.equal(u.view(torch.int16), v.view(torch.int16))
        ref = oracle_layer(oracle, li, 12, eps=1e-6).prefill(li.x.astype(np.float64))
        cur = error_curves(li.x.astype(np.float64), ref, tuple(tio.to_host(t) for t in a))
        for name in ("y", "K", "V"):
            assert cur[name].max() <= TOL["bf16"]
    finally:
        ctx.rt_destroy()


def test_persistent_bounded_wait_expires_cleanly(monkeypatch):
    """A spin limit of one poll forces the kernel's own bounded waits to give up: every workgroup exits,
    the host reports it, and the context refuses further work."""
    binding, tio = _gpu()
    monkeypatch.setenv("RT_SPIN_LIMIT", "1")
    li = gen.make_custom(4, "bf16", 2, 64, 256, 4, 1024)
    ctx = binding.RTContext(256, 4, 1024, 2, 64, "bf16", flags=binding.RT_FLAG_ENGINE_PERSISTENT)
    monkeypatch.delenv("RT_SPIN_LIMIT")
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
        xd = tio.to_device(li.x, "bf16")
        tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        assert ctx.device_wait_expired() == 1
        y = torch.empty_like(xd)
        K = torch.zeros((64, 2, 4, 64), dtype=xd.dtype, device=xd.device)
        assert ctx.raw_prefill(dl.struct, xd.data_ptr(), 2, 64, y.data_ptr(), K.data_ptr(), torch.zeros_like(K).data_ptr(),
                               64) == binding.RT_ERR_STATE
    finally:
        ctx.rt_destroy()


# ----------------------------------------------------------------------------- prefill == decode
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefill_then_decode_matches_oracle_and_full_prefill(oracle, dtype):
    binding, tio = _gpu()
    B, N, d, H, F, n0 = 3, 300, 128, 2, 512, 270
    li = gen.make_custom(9, dtype, B, N, d, H, F, gains="random")
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, H, alpha=0.8).prefill(x64)
    ctx = binding.RTContext(d, H, F, B, N, dtype, resid_scale=0.8, flags=binding.RT_FLAG_ENGINE_STEPWISE)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, dtype)
        xd = tio.to_device(li.x, dtype)
        y0, K, V = tio.prefill(ctx, dl, xd[:, :n0].contiguous(), kv_cap=N)
        ys = [y0]
        for t in range(n0, N):
            y_t = torch.empty((B, d), dtype=xd.dtype, device=xd.device)
            ctx.rt_decode_step(dl.struct, xd[:, t].contiguous(), t, y_t, K, V)
            ys.append(y_t[:, None])
        torch.cuda.synchronize()
        got = (tio.to_host(torch.cat(ys, dim=1)), tio.to_host(K), tio.to_host(V))
        # decode from an empty cache as well: N' successive steps equal a prefill of length N'
        K2 = torch.zeros_like(K)
        V2 = torch.zeros_like(V)
        y2 = []
        for t in range(12):
            y_t = torch.empty((B, d), dtype=xd.dtype, device=xd.device)
            ctx.rt_decode_step(dl.struct, xd[:, t].contiguous(), t, y_t, K2, V2)
            y2.append(y_t[:, None])
        torch.cuda.synchronize()
        got2 = tio.to_host(torch.cat(y2, dim=1))
    finally:
        ctx.rt_destroy()
    cur = error_curves(x64, ref, got)
    print("\n  [prefill+decode %s] %s" % (dtype, summarize(cur)))
    for name in ("y", "K", "V"):
        assert cur[name].max() <= TOL[dtype]
    from tests.parity_util import rel_err_rows
    assert rel_err_rows(got2, ref[0][:, :12]).max() <= TOL[dtype]


# ----------------------------------------------------------------------------- error paths (host side only)
def test_invalid_arguments_are_rejected_before_any_launch():
    binding, tio = _gpu()
    with pytest.raises(binding.RTError):
        binding.RTContext(128, 2, 512, 1, 16, "f32", p_min=3)
    with pytest.raises(binding.RTError):
        binding.RTContext(96, 2, 512, 1, 16, "f32")                       # head_dim 48
    with pytest.raises(binding.RTError):
        binding.RTContext(128, 2, 512, 1, 16, "bf16", p_min=8)            # MFMA path needs p_min >= 32
    ctx = binding.RTContext(128, 2, 512, 2, 16, "f32", flags=binding.RT_FLAG_ENGINE_STEPWISE)
    try:
        li = gen.make_custom(3, "f32", 2, 16, 128, 2, 512)
        dl = tio.DeviceLayer(li.weights, li.gains, "f32")
        x = tio.to_device(li.x, "f32")
        y = torch.full_like(x, 7.0)
        K = torch.zeros((16, 2, 2, 64), device=x.device)
        V = torch.zeros_like(K)
        P = lambda t: t.data_ptr()
        assert ctx.raw_prefill(dl.struct, P(x), 3, 16, P(y), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG   # B > max
        assert ctx.raw_prefill(dl.struct, P(x), 2, 17, P(y), P(K), P(V), 17) == binding.RT_ERR_INVALID_ARG   # N > max
        assert ctx.raw_prefill(dl.struct, P(x), 2, 16, P(y), P(K), P(V), 15) == binding.RT_ERR_INVALID_ARG   # kv_cap < N
        assert ctx.raw_prefill(dl.struct, P(x), 2, 16, P(x), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG   # y aliases x
        assert ctx.raw_prefill(dl.struct, 0, 2, 16, P(y), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG      # null x
        assert ctx.raw_prefill(None, P(x), 2, 16, P(y), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG        # null weights
        assert "overlap" in ctx.last_error() or ctx.last_error()
        assert ctx.raw_decode(dl.struct, P(x), 2, 16, P(y), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG    # t >= kv_cap
        assert ctx.raw_decode(dl.struct, P(x), 2, -1, P(y), P(K), P(V), 16) == binding.RT_ERR_INVALID_ARG
        torch.cuda.synchronize()
        assert float(y.min()) == 7.0 and float(K.abs().max()) == 0.0      # outputs untouched
    finally:
        ctx.rt_destroy()


def test_two_runs_are_bit_identical(oracle):
    binding, tio = _gpu()
    li = gen.make_custom(4, "bf16", 2, 160, 256, 4, 1024)
    ctx = binding.RTContext(256, 4, 1024, 2, 160, "bf16", flags=binding.RT_FLAG_ENGINE_STEPWISE)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
        xd = tio.to_device(li.x, "bf16")
        a = tio.prefill(ctx, dl, xd)
        b = tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        for u, v in zip(a, b):
            assert torch.equal(u.view(torch.int16), v.view(torch.int16))
    finally:
        ctx.rt_destroy()
