"""Every schedule with its partial softmax states poisoned (RT_FLAG_DEBUG_POISON: all stored (m, l, o) triples are NaN
when a prefill starts): one oracle-parity run per engine.  A state that a schedule reads before the same call has
written it - Algorithm 1 as printed, the persistent engine's shifted blocks, the chunked schedule of the layer
wavefront, the blocked recurrence - would reach y, K or V as NaN and fail the comparison."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, oracle_layer
from tests.test_gpu_parity import _run_case
from tests.test_gpu_stack import _run_elementwise, EMB_UNIT
from tests.test_gpu_parallel import _setup, _check

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _b():
    from paper_2604_21215_amd import binding
    return binding


def test_poisoned_states_stepwise_fp32(oracle):
    b = _b()
    _run_case(oracle, "f32", 2, 333, 128, 2, 512, p_min=4, flags=b.RT_FLAG_DEBUG_POISON | b.RT_FLAG_ENGINE_STEPWISE,
              expect_engine="stepwise")


def test_poisoned_states_stepwise_bf16_matrix_core_tiles(oracle):
    b = _b()
    _run_case(oracle, "bf16", 2, 300, 256, 4, 1024, flags=b.RT_FLAG_DEBUG_POISON | b.RT_FLAG_ENGINE_STEPWISE,
              expect_engine="stepwise")


def test_poisoned_states_persistent_engine(oracle):
    b = _b()
    _run_case(oracle, "bf16", 3, 700, 256, 4, 1024, flags=b.RT_FLAG_DEBUG_POISON | b.RT_FLAG_ENGINE_PERSISTENT,
              expect_engine="persistent")


@pytest.mark.parametrize("dtype,N,chunk,p_min", [("f32", 130, 16, 4), ("bf16", 300, 64, 0)])
def test_poisoned_states_layer_wavefront(oracle, dtype, N, chunk, p_min):
    wl = gen.Workload("stack_poison", dtype, 2, N, 256 if dtype == "bf16" else 128, 4 if dtype == "bf16" else 2,
                      1024 if dtype == "bf16" else 512, layers=3, vocab=300, decode_steps=2, seed=996)
    _run_elementwise(oracle, wl, 2, N, 2, flags=_b().RT_FLAG_DEBUG_POISON, emb_scale=EMB_UNIT, wavefront=True, chunk=chunk,
                     p_min=p_min)


def test_poisoned_states_blocked_recurrence(oracle):
    B, N, d, H, F, block = 2, 300, 256, 4, 1024, 8
    li = gen.make_custom(27, "bf16", B, N, d, H, F)
    x64 = li.x.astype(np.float64)
    ref = oracle_layer(oracle, li, H, eps=1e-6).prefill_blocked(x64, block)
    ctx, tio, dl, xd, y, K, V = _setup(li, B, N, d, H, F, rms_eps=1e-6, flags=_b().RT_FLAG_DEBUG_POISON)
    try:
        ctx.rt_layer_prefill_blocked(dl.struct, xd, block, y, K, V)
        torch.cuda.synchronize()
        _check("blocked recurrence, poisoned states", x64, ref, (tio.to_host(y), tio.to_host(K), tio.to_host(V)), TOL["bf16"])
    finally:
        ctx.rt_destroy()
