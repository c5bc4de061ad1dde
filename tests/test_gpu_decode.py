"""The single-launch decoding step (one cooperative kernel per rt_decode_step: bf16 storage, d a multiple of 256,
F = 4 d, B H <= 256) against the CPU oracle's prefill of the same sequence, position by position: from a cache the
prefill engine left, from an empty cache, over caches short and long enough to give a wavefront zero, one and several
64-key chunks, with gains, ALiBi, the norm-free layer and a scaled residual.  The multi-launch step (the path every
other shape takes) runs beside it on the same inputs."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, rel_err_rows, oracle_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _decode_case(oracle, B, N, d, H, *, n0, steps, seed, gains="random", alpha=1.0, scale=1.0, alibi=0.0, flags=0, max_batch=None):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    F = 4 * d
    assert list(steps) == list(range(n0, n0 + len(steps))) and steps[-1] < N
    li = gen.make_custom(seed, "bf16", B, N, d, H, F, gains=gains)
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, H, alpha=alpha, attn_scale=scale, eps=1e-6, alibi_max_bias=alibi,
                       **({"norm_free": True} if flags & 1 else {})).prefill(x64)
    worst = {}
    for name, extra in (("single-launch", 0), ("multi-launch", binding.RT_FLAG_ENGINE_STEPWISE)):
        ctx = binding.RTContext(d, H, F, max_batch or B, N, "bf16", resid_scale=alpha, attn_scale=scale, rms_eps=1e-6,
                                flags=flags | extra, alibi_max_bias=alibi)
        try:
            dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
            xd = tio.to_device(li.x, "bf16")
            K = torch.zeros((N, B, H, 64), dtype=xd.dtype, device=xd.device)
            V = torch.zeros_like(K)
            if n0 > 0:
                y0 = torch.empty((B, n0, d), dtype=xd.dtype, device=xd.device)
                ctx.rt_layer_prefill(dl.struct, xd[:, :n0].contiguous(), y0, K, V)
            ey = ek = ev = 0.0
            for t in steps:   # consecutive from n0: every step reads the rows the prefill and the steps before it wrote
                y_t = torch.full((B, d), 7.0, dtype=xd.dtype, device=xd.device)
                ctx.rt_decode_step(dl.struct, xd[:, t].contiguous(), t, y_t, K, V)
                torch.cuda.synchronize()
                assert ctx.device_wait_expired() == 0
                if not extra:
                    assert ctx.engine_name() == "decode-single-launch"
                ey = max(ey, rel_err_rows(tio.to_host(y_t), ref[0][:, t]).max())
                ek = max(ek, rel_err_rows(tio.to_host(K[t]), ref[1][t]).max())
                ev = max(ev, rel_err_rows(tio.to_host(V[t]), ref[2][t]).max())
            if steps[-1] + 1 < N:   # cache rows after the last decoded position are untouched
                assert float(K[steps[-1] + 1:].abs().max()) == 0.0 and float(V[steps[-1] + 1:].abs().max()) == 0.0
            worst[name] = (ey, ek, ev)
        finally:
            ctx.rt_destroy()
    print("\n  [decode B=%d d=%d H=%d steps %s..%s] " % (B, d, H, steps[0], steps[-1]) +
          "; ".join("%s y %.1e K %.1e V %.1e" % (k, *v) for k, v in worst.items()))
    for k, v in worst.items():
        assert max(v) <= TOL["bf16"], (k, v)


def test_decode_from_empty_cache_and_short_caches(oracle):
    # t = 0 (no cached key), 1, and across the first chunk boundary
    _decode_case(oracle, 3, 70, 256, 4, n0=0, steps=list(range(0, 70)), seed=31)


def test_decode_after_prefill_small_width(oracle):
    # B H = 12: sixteen workgroups share each (b, h); most wavefronts hold no chunk
    _decode_case(oracle, 3, 300, 256, 4, n0=260, steps=list(range(260, 300)), seed=32, alpha=0.8, scale=0.5)


def test_decode_full_batch_many_heads(oracle):
    # B H = 128 at d = 512: two workgroups per (b, h); max_batch 16 sizes the staging rows
    _decode_case(oracle, 16, 200, 512, 8, n0=190, steps=list(range(190, 200)), seed=33)


def test_decode_three_quarter_width(oracle):
    _decode_case(oracle, 5, 150, 768, 12, n0=140, steps=list(range(140, 150)), seed=34, gains="unit")


def test_decode_headline_width_long_cache(oracle):
    # d = 1024, B = 8: sixteen workers per (b, h), 1200 keys: wavefronts with one and with two chunks
    _decode_case(oracle, 8, 1203, 1024, 16, n0=1196, steps=list(range(1196, 1203)), seed=35, gains="unit")


def test_decode_alibi_and_norm_free(oracle):
    _decode_case(oracle, 2, 200, 256, 4, n0=180, steps=list(range(180, 200)), seed=36, alibi=8.0)
    _decode_case(oracle, 2, 100, 256, 4, n0=90, steps=list(range(90, 100)), seed=37, flags=1, scale=0.125)


def test_decode_smaller_batch_than_context(oracle):
    _decode_case(oracle, 2, 150, 512, 8, n0=130, steps=list(range(130, 140)), seed=38, max_batch=8)   # rows 140 .. 149 stay untouched


def test_decode_many_chunks_per_wavefront(oracle, monkeypatch):
    # one workgroup per (b, h) (RT_DECODE_SPLIT = 1): 23 chunks over eight wavefronts - the loop that reloads a
    # wavefront's two chunk buffers runs, some wavefronts end on the first buffer and some on the second
    monkeypatch.setenv("RT_DECODE_SPLIT", "1")
    _decode_case(oracle, 3, 1450, 256, 4, n0=1444, steps=list(range(1444, 1450)), seed=39, scale=0.5)


def test_decode_largest_layout(oracle):
    # B H = 256 at d = 1024: one workgroup per (b, h), sixteen staged rows - the largest LDS layout the kernel has
    _decode_case(oracle, 16, 75, 1024, 16, n0=70, steps=list(range(70, 75)), seed=40, gains="unit")


def test_decode_batches_beyond_the_single_launch_run_in_chunks(oracle):
    # 40 sequences: three launches of 16 + 16 + 8 rows, each on its slice of the position-major cache rows (row stride of the
    # whole batch); 20 at the headline width: 16 + 4
    _decode_case(oracle, 40, 70, 256, 4, n0=64, steps=list(range(64, 70)), seed=41, scale=0.5, alibi=8.0)
    _decode_case(oracle, 20, 40, 1024, 16, n0=36, steps=list(range(36, 40)), seed=42, scale=0.25)
