"""rt_decode_step_static (the decoding step for callers that cannot allocate: no context, scratch in a static device
array) against rt_decode_step on the same inputs, through the C ABI: bit for bit, on two calls in a row of which the
second is smaller (fewer sequences, an earlier position), for the matrix-core and the plain-ALU kernels."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _bits(t):
    return t.contiguous().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.mark.parametrize("dtype,d,H,F", [("bf16", 256, 4, 1024), ("f32", 128, 2, 512), ("bf16", 192, 3, 768)])
def test_static_decode_matches_context_decode(dtype, d, H, F):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding, torch_io as tio
    Bmax, N, cap = 3, 150, 160
    li = gen.make_custom(4242, dtype, Bmax, N + 1, d, H, F, gains="random")
    stream = torch.cuda.current_stream().cuda_stream
    ctx = binding.RTContext(d, H, F, Bmax, cap, dtype, rms_eps=1e-6, attn_scale=0.5, stream=stream,
                            flags=binding.RT_FLAG_ENGINE_STEPWISE)   # the multi-launch step: the kernels the context-free call runs
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, dtype)
        xd = tio.to_device(li.x, dtype)
        # two (B, t) cases in a row, the second smaller in both; each from a cache the prefill engine wrote
        for B, t in ((3, 150), (2, 70)):
            xb = xd[:B].contiguous()
            y = torch.empty((B, t, d), dtype=xd.dtype, device=xd.device)
            K = torch.zeros((cap, B, H, 64), dtype=xd.dtype, device=xd.device)
            V = torch.zeros_like(K)
            ctx.rt_layer_prefill(dl.struct, xb[:, :t].contiguous(), y, K, V)
            x_t = xb[:, t].contiguous()
            K1, V1, K2, V2 = K.clone(), V.clone(), K.clone(), V.clone()
            y1 = torch.empty((B, d), dtype=xd.dtype, device=xd.device)
            y2 = torch.full_like(y1, 7.0)
            ctx.rt_decode_step(dl.struct, x_t, t, y1, K1, V1)
            binding.rt_decode_step_static(ctx.cfg, dl.struct, x_t, t, y2, K2, V2)
            torch.cuda.synchronize()
            assert ctx.device_wait_expired() == 0
            np.testing.assert_array_equal(_bits(y2), _bits(y1))
            np.testing.assert_array_equal(_bits(K2), _bits(K1))
            np.testing.assert_array_equal(_bits(V2), _bits(V1))
            assert np.abs(tio.to_host(y1)).max() > 0 and np.abs(tio.to_host(K1[t])).max() > 0
    finally:
        ctx.rt_destroy()


def test_static_decode_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from paper_2604_21215_amd import binding
    cfg = binding.rt_config(1024, 16, 64, 4096, 8, 1 << 16, binding.RT_BF16, 0, 1.0, 1.0, 1e-6, 0, 0, None, 0.0)
    w = binding.rt_layer_weights(*([1 << 30] * 6))
    fake = [(i + 1) << 42 for i in range(4)]
    # 8 sequences x 16 heads x 313 splits of partial states: more than the static array holds
    rc = binding.raw_decode_static(cfg, w, fake[0], 8, 20000, fake[1], fake[2], fake[3], 20001)
    assert rc == binding.RT_ERR_INVALID_ARG
    assert b"static scratch holds" in binding.load().rt_last_error(None)
    rc = binding.raw_decode_static(cfg, w, fake[0], 9, 100, fake[1], fake[2], fake[3], 20001)   # B > max_batch
    assert rc == binding.RT_ERR_INVALID_ARG
    rc = binding.raw_decode_static(cfg, w, fake[0], 8, 100, fake[0], fake[2], fake[3], 20001)   # y_t aliases x_t
    assert rc == binding.RT_ERR_INVALID_ARG
