"""Seeded sweep over shapes and options the hand-picked parity cases do not name: widths 128 .. 1024, batch 1 .. 16,
lengths around the block boundaries of Algorithm 1 (31 .. 385), gains, residual and logit scales, positional bias,
threshold p_min and cache rows beyond N, each compared with the fp64 oracle exactly as the named cases are (forward:
y, K, V per position plus two decoding steps over the cache; backward: dx and every parameter gradient).  The draws
are fixed by the seed, so every run checks the same cases."""
import numpy as np
import pytest

from tests import test_gpu_backward as bw
from tests import test_gpu_parity as fw

pytestmark = pytest.mark.gpu

LENGTHS = [1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200, 257, 300, 385]


def _forward_cases(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        d = int(rng.choice([128, 256, 512, 768, 1024]))
        F = 4 * d if rng.random() < 0.8 else 2 * d
        B, N = int(rng.integers(1, 17)), int(rng.choice(LENGTHS))
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        if dtype == "f32":          # the plain-ALU engine: keep the oracle and the GPU to a second per case
            N, B = min(N, 130), min(B, 4)
        kw = dict(gains=str(rng.choice(["unit", "random"])), seed=int(rng.integers(1, 10000)),
                  alpha=float(rng.choice([1.0, 0.7, 0.3])), scale=float(rng.choice([1.0, 0.5, 0.125])),
                  alibi=float(rng.choice([0.0, 0.0, 8.0])), n_decode=min(2, N), p_min=int(rng.choice([0, 0, 0, 32, 64])))
        if N > 1 and rng.random() < 0.3:
            kw["kv_cap"] = N + int(rng.integers(1, 70))
        yield dtype, B, N, d, d // 64, F, kw


def _backward_cases(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        d = int(rng.choice([128, 256, 512, 768, 1024]))
        B, N = int(rng.integers(1, 9)), int(rng.choice([1, 2, 31, 33, 64, 65, 97, 130]))
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        if dtype == "f32":
            d = min(d, 256)
        kw = dict(gains="random", alpha=float(rng.choice([1.0, 0.7])), scale=float(rng.choice([0.5, 0.25, 0.125])),
                  alibi=float(rng.choice([0.0, 8.0])), seed=int(rng.integers(1, 10000)),
                  shared_kv_gain=bool(rng.random() < 0.3), with_pair_grads=bool(rng.random() < 0.7))
        yield dtype, B, N, d, d // 64, 4 * d, kw


@pytest.mark.parametrize("seed", [11, 12])
def test_forward_and_decoding_step_on_drawn_shapes(oracle, seed):
    for dtype, B, N, d, H, F, kw in _forward_cases(seed, 24):
        print("\n  case: %s B=%d N=%d d=%d F=%d %s" % (dtype, B, N, d, F, kw), flush=True)
        fw._run_case(oracle, dtype, B, N, d, H, F, **kw)


@pytest.mark.parametrize("seed", [21])
def test_backward_on_drawn_shapes(oracle, seed):
    for dtype, B, N, d, H, F, kw in _backward_cases(seed, 12):
        print("\n  case: %s B=%d N=%d d=%d %s" % (dtype, B, N, d, kw), flush=True)
        bw._run(oracle, dtype, B, N, d, H, F, **kw)
