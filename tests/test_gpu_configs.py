"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times
(default engine selection, default p_min), element by element against the CPU oracle."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, error_curves, summarize, oracle_layer

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
    return cur


def test_config1_fp32_full(oracle):
    cur = _full(oracle, "cfg1", engine="stepwise")
    assert cur["branch"].max() < 1e-4


def test_config2_bf16_full(oracle):
    _full(oracle, "cfg2")


def test_config3_bf16_full_headline(oracle):
    _full(oracle, "cfg3")


@pytest.mark.parametrize("N", [1024, 2048, 4096, 8192])
def test_config4_sweep_prefixes(oracle, N):
    _full(oracle, "cfg4_8192", N=N)
