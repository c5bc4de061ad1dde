"""GPU parity of the loop-free evaluations against the CPU oracle: rt_layer_recompute (the layer with its output
given, Sec. 6.1) and rt_transformer_layer (Sec. 2.1), bf16 storage, element by element as error curves over position
(tolerance 2e-2 per position for y, K, V)."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, error_curves, summarize, oracle_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _setup(li, B, N, d, H, F, **kw):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    ctx = binding.RTContext(d, H, F, B, N, "bf16", stream=torch.cuda.current_stream().cuda_stream, **kw)
    dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
    xd = tio.to_device(li.x, "bf16")
    y = torch.empty_like(xd)
    K = torch.zeros((N, B, H, d // H), dtype=xd.dtype, device=xd.device)
    V = torch.zeros_like(K)
    return ctx, tio, dl, xd, y, K, V


def _check(name, x64, ref, got, tol):
    cur = error_curves(x64, ref, got)
    print("\n  [%s] %s" % (name, summarize(cur)))
    for k in ("y", "K", "V"):
        assert cur[k].max() <= tol, "%s %s: %.3e at position %d" % (name, k, cur[k].max(), int(np.argmax(cur[k])))


@pytest.mark.parametrize("B,N,d,H,F,alibi,gains,alpha,scale", [
    (2, 200, 256, 4, 1024, 0.0, "unit", 1.0, 1.0),
    (3, 333, 320, 5, 1280, 8.0, "random", 0.7, 0.5),       # odd head count, ragged N, bias, gains
    (2, 700, 1024, 16, 4096, 0.0, "unit", 1.0, 1.0),       # blocks up to 512 keys, several query workgroups
    (1, 33, 256, 4, 1024, 0.0, "unit", 1.0, 1.0),
    (5, 600, 256, 4, 1024, 0.0, "random", 0.7, 1.0),       # 3000 rows: the LDS-tiled products, ragged last row tile
])
def test_recompute_from_exact_output(oracle, B, N, d, H, F, alibi, gains, alpha, scale):
    """z = the oracle's output (rounded to bf16): the recompute must reproduce the oracle's y, K, V."""
    li = gen.make_custom(21, "bf16", B, N, d, H, F, gains=gains)
    x64 = li.x.astype(np.float64)
    lay = oracle_layer(oracle, li, H, alpha=alpha, attn_scale=scale, eps=1e-6, alibi_max_bias=alibi)
    ref = lay.prefill(x64)
    ctx, tio, dl, xd, y, K, V = _setup(li, B, N, d, H, F, resid_scale=alpha, attn_scale=scale, rms_eps=1e-6, alibi_max_bias=alibi)
    try:
        zd = tio.to_device(gen.round_to_bf16(ref[0].astype(np.float32)), "bf16")
        ctx.rt_layer_recompute(dl.struct, xd, zd, y, K, V)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "recompute"
        _check("recompute B=%d N=%d d=%d alibi=%g" % (B, N, d, alibi), x64, ref, (tio.to_host(y), tio.to_host(K), tio.to_host(V)),
               TOL["bf16"])
    finally:
        ctx.rt_destroy()


def test_recompute_of_an_arbitrary_z_and_of_the_prefill_output(oracle):
    """(1) z that is NOT the layer's output: the recompute is still a defined map (K, V from z, y from x and those) and must
    match the oracle's recompute of the same z; (2) z = what rt_layer_prefill produced on the GPU: y reproduces it and
    K, V equal the prefill's up to rounding."""
    B, N, d, H, F = 2, 300, 256, 4, 1024
    li = gen.make_custom(22, "bf16", B, N, d, H, F)
    x64 = li.x.astype(np.float64)
    lay = oracle_layer(oracle, li, H, eps=1e-6)
    z = gen.round_to_bf16((li.x + 0.5 * gen.make_custom(23, "bf16", B, N, d, H, F).x).astype(np.float32))
    ref = lay.recompute(x64, z.astype(np.float64))
    ctx, tio, dl, xd, y, K, V = _setup(li, B, N, d, H, F, rms_eps=1e-6)
    try:
        ctx.rt_layer_recompute(dl.struct, xd, tio.to_device(z, "bf16"), y, K, V)
        torch.cuda.synchronize()
        _check("recompute of an arbitrary z", x64, ref, (tio.to_host(y), tio.to_host(K), tio.to_host(V)), TOL["bf16"])
        y1, K1, V1 = tio.prefill(ctx, dl, xd)
        torch.cuda.synchronize()
        y2, K2, V2 = torch.empty_like(y1), torch.zeros_like(K1), torch.zeros_like(V1)
        ctx.rt_layer_recompute(dl.struct, xd, y1, y2, K2, V2)
        torch.cuda.synchronize()
        _check("recompute of the prefill's own output", x64, (tio.to_host(y1), tio.to_host(K1), tio.to_host(V1)),
               (tio.to_host(y2), tio.to_host(K2), tio.to_host(V2)), TOL["bf16"])
    finally:
        ctx.rt_destroy()


@pytest.mark.parametrize("B,N,d,H,F,alibi", [(2, 200, 256, 4, 1024, 0.0), (3, 333, 320, 5, 1280, 8.0), (2, 600, 1024, 16, 4096, 0.0),
                                               (6, 450, 384, 6, 1536, 0.0),    # 2700 rows: the LDS-tiled products
                                               (2, 1, 256, 4, 1024, 0.0),      # a single position: only the temporary pair
                                               (2, 128, 256, 4, 1024, 8.0),    # exactly one query tile of the masked pass
                                               (2, 129, 256, 4, 1024, 8.0)])   # ... and one position more
def test_transformer_layer(oracle, B, N, d, H, F, alibi):
    li = gen.make_custom(24, "bf16", B, N, d, H, F, gains="random")
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, H, alpha=0.8, eps=1e-6, alibi_max_bias=alibi).transformer(x64)
    ctx, tio, dl, xd, y, K, V = _setup(li, B, N, d, H, F, resid_scale=0.8, rms_eps=1e-6, alibi_max_bias=alibi)
    try:
        ctx.rt_transformer_layer(dl.struct, xd, y, K, V)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "transformer"
        _check("transformer layer B=%d N=%d d=%d alibi=%g" % (B, N, d, alibi), x64, ref[:3],
               (tio.to_host(y), tio.to_host(K), tio.to_host(V)), TOL["bf16"])
    finally:
        ctx.rt_destroy()


@pytest.mark.parametrize("B,N,d,H,F,block,p_min,alibi", [
    (2, 200, 256, 4, 1024, 8, 32, 0.0),
    (3, 333, 320, 5, 1280, 32, 32, 8.0),      # block = p_min, ragged last block, bias
    (2, 300, 256, 4, 1024, 1, 32, 0.0),       # one position per block: the RT layer itself
    (8, 400, 1024, 16, 4096, 16, 64, 0.0),
])
def test_blocked_recurrence(oracle, B, N, d, H, F, block, p_min, alibi):
    """rt_layer_prefill_blocked against the oracle's blocked recurrence (persistent pairs across blocks, temporary pairs
    inside a block)."""
    li = gen.make_custom(26, "bf16", B, N, d, H, F, gains="random")
    x64 = li.x.astype(np.float64)
    lay = oracle_layer(oracle, li, H, alpha=0.8, eps=1e-6, alibi_max_bias=alibi)
    ref = lay.prefill_blocked(x64, block)
    ctx, tio, dl, xd, y, K, V = _setup(li, B, N, d, H, F, resid_scale=0.8, rms_eps=1e-6, alibi_max_bias=alibi, p_min=p_min)
    try:
        ctx.rt_layer_prefill_blocked(dl.struct, xd, block, y, K, V)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "blocked"
        _check("blocked recurrence B=%d N=%d d=%d block=%d" % (B, N, d, block), x64, ref,
               (tio.to_host(y), tio.to_host(K), tio.to_host(V)), TOL["bf16"])
        if block == 1:       # the same layer as rt_layer_prefill evaluates
            y1, K1, V1 = tio.prefill(ctx, dl, xd)
            torch.cuda.synchronize()
            _check("block = 1 against rt_layer_prefill", x64, (tio.to_host(y1), tio.to_host(K1), tio.to_host(V1)),
                   (tio.to_host(y), tio.to_host(K), tio.to_host(V)), TOL["bf16"])
        from paper_2604_21215_amd import binding
        with pytest.raises(binding.RTError):
            ctx.rt_layer_prefill_blocked(dl.struct, xd, 2 * p_min, y, K, V)      # block > p_min
        with pytest.raises(binding.RTError):
            ctx.rt_layer_prefill_blocked(dl.struct, xd, 3, y, K, V)              # not a power of two
    finally:
        ctx.rt_destroy()


def test_parallel_entry_points_reject_what_they_do_not_cover():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    li = gen.make_custom(25, "f32", 1, 16, 128, 2, 512)
    ctx = binding.RTContext(128, 2, 512, 1, 16, "f32")
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, "f32")
        xd = tio.to_device(li.x, "f32")
        y, K, V = torch.empty_like(xd), torch.zeros((16, 1, 2, 64), device=xd.device), torch.zeros((16, 1, 2, 64), device=xd.device)
        with pytest.raises(binding.RTError) as ei:
            ctx.rt_layer_prefill_blocked(dl.struct, xd, 3, y, K, V)       # not a power of two
        assert ei.value.status == "RT_ERR_INVALID_ARG"
        with pytest.raises(binding.RTError):
            ctx.rt_layer_recompute(dl.struct, xd, xd, xd, K, V)          # output overlaps an input
        with pytest.raises(binding.RTError):
            ctx.rt_transformer_layer(dl.struct, xd, y, K, K)             # K and V overlap
    finally:
        ctx.rt_destroy()


@pytest.mark.parametrize("dtype,B,N,d,H,F,alibi,flags", [
    ("f32", 1, 256, 128, 2, 512, 0.0, 0),            # the fp32 benchmark configuration's shape
    ("f32", 3, 77, 192, 3, 768, 8.0, 0),             # ragged, odd head count, bias
    ("bf16", 2, 150, 256, 4, 1024, 0.0, "no_mfma"),  # bf16 storage without the matrix-core kernels
])
def test_loop_free_layers_on_the_plain_alu_kernels(oracle, dtype, B, N, d, H, F, alibi, flags):
    """fp32 storage (tolerance 1e-4) and bf16 without the MFMA kernels: rt_transformer_layer against the oracle's
    Transformer layer; rt_layer_recompute fed with the oracle's output (rounded to the storage type) against the
    oracle's prefill, and fed with an arbitrary z against the oracle's recompute of the same z; rt_layer_prefill_blocked
    against the oracle's blocked recurrence (blocks of 1, the RT layer itself, and of 8)."""
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    li = gen.make_custom(31, dtype, B, N, d, H, F, gains="random")
    x64 = li.x.astype(np.float64)
    lay = oracle_layer(oracle, li, H, alpha=0.9, eps=1e-6, alibi_max_bias=alibi)
    kw = dict(resid_scale=0.9, rms_eps=1e-6, alibi_max_bias=alibi, stream=torch.cuda.current_stream().cuda_stream)
    if flags == "no_mfma":
        kw["flags"] = binding.RT_FLAG_NO_MFMA
    ctx = binding.RTContext(d, H, F, B, N, dtype, **kw)
    tol = TOL[dtype]
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, dtype)
        xd = tio.to_device(li.x, dtype)
        y = torch.empty_like(xd)
        K = torch.zeros((N, B, H, d // H), dtype=xd.dtype, device=xd.device)
        V = torch.zeros_like(K)
        got = lambda: (tio.to_host(y), tio.to_host(K), tio.to_host(V))
        ctx.rt_transformer_layer(dl.struct, xd, y, K, V)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "transformer"
        _check("plain-ALU Transformer layer %s B=%d N=%d" % (dtype, B, N), x64, lay.transformer(x64), got(), tol)
        ref = lay.prefill(x64)
        z = ref[0].astype(np.float32)
        if dtype == "bf16":
            z = gen.round_to_bf16(z)
        ctx.rt_layer_recompute(dl.struct, xd, tio.to_device(z, dtype), y, K, V)
        torch.cuda.synchronize()
        assert ctx.engine_name() == "recompute"
        _check("plain-ALU recompute from the exact output %s" % dtype, x64, ref, got(), tol)
        z2 = (li.x + 0.5 * gen.make_custom(32, dtype, B, N, d, H, F).x).astype(np.float32)
        if dtype == "bf16":
            z2 = gen.round_to_bf16(z2)
        ctx.rt_layer_recompute(dl.struct, xd, tio.to_device(z2, dtype), y, K, V)
        torch.cuda.synchronize()
        _check("plain-ALU recompute of an arbitrary z %s" % dtype, x64, lay.recompute(x64, z2.astype(np.float64)), got(), tol)
        for block in (1, 8):
            ctx.rt_layer_prefill_blocked(dl.struct, xd, block, y, K, V)
            torch.cuda.synchronize()
            assert ctx.engine_name() == "blocked"
            _check("plain-ALU blocked recurrence (%d) %s" % (block, dtype), x64, lay.prefill_blocked(x64, block), got(), tol)
    finally:
        ctx.rt_destroy()
