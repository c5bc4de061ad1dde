"""GPU parity of rt_layer_backward (Sec. 6.4) against the fp64 backward oracle (oracle/rt_backward.py, itself pinned by
central differences of the forward oracle): dx as an error curve over position, every parameter gradient norm-wise.
Tolerances: 1e-4 for fp32 storage, 2e-2 for bf16 storage."""
import numpy as np
import pytest

from paper_2604_21215_amd import inputs as gen
from tests.parity_util import TOL, rel_err_rows

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

MATS = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")
GAINS = ("g_attn", "g_mlp", "g_kv", "g_q", "g_k")


def _run(oracle, dtype, B, N, d, H, F, *, gains="random", alpha=1.0, scale=1.0, alibi=0.0, seed=31, shared_kv_gain=False,
         norm_free=False, with_pair_grads=True, z_from_gpu=False, tol=None, no_mfma=False):
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible")
    from oracle import rt_backward as bwd
    from paper_2604_21215_amd import binding, torch_io as tio
    li = gen.make_custom(seed, dtype, B, N, d, H, F, gains=gains)
    w = {k: v.astype(np.float64) for k, v in li.weights.items()}
    g = {k: v.astype(np.float64) for k, v in li.gains.items()}
    if shared_kv_gain:
        g["g_kv"] = None
    x = li.x.astype(np.float64)
    kw = dict(alpha=alpha, attn_scale=scale, eps=1e-6, alibi_max_bias=alibi)
    store = (lambda a: gen.round_to_bf16(a.astype(np.float32))) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    lay = oracle.Layer(w, H, gains={k: (g["g_attn"] if (k == "g_kv" and v is None) else v) for k, v in g.items()},
                       norm_free=norm_free, **kw)
    z = store(lay.prefill(x)[0])                       # the layer's output as the caller would hold it
    rng = np.random.default_rng(seed + 1000)
    gy = store(rng.standard_normal((B, N, d)))
    gK = store(rng.standard_normal((N, B, H, d // H))) if with_pair_grads else None
    gV = store(rng.standard_normal((N, B, H, d // H))) if with_pair_grads else None

    flags = (binding.RT_FLAG_NORM_FREE if norm_free else 0) | (binding.RT_FLAG_NO_MFMA if no_mfma else 0)
    ctx = binding.RTContext(d, H, F, B, N, dtype, resid_scale=alpha, attn_scale=scale, rms_eps=1e-6, alibi_max_bias=alibi,
                            flags=flags, stream=torch.cuda.current_stream().cuda_stream)
    try:
        dl = tio.DeviceLayer(li.weights, li.gains, dtype, alias_kv_gain=shared_kv_gain)
        xd = tio.to_device(li.x, dtype)
        if z_from_gpu:                                 # the whole pipeline on the GPU: forward, then backward from its output
            y, _, _ = tio.prefill(ctx, dl, xd)
            zd = y
        else:
            zd = tio.to_device(z, dtype)
        dev = lambda a: None if a is None else tio.to_device(a, dtype)
        dx = torch.empty((B, N, d), dtype=torch.float32, device="cuda:0")
        grads = {k: torch.full(tuple(li.weights[k].shape), float("nan"), dtype=torch.float32, device="cuda:0") for k in MATS}
        grads.update({k: torch.full((d,), float("nan"), dtype=torch.float32, device="cuda:0") for k in GAINS})
        ctx.rt_layer_backward(dl.struct, xd, zd, dev(gy), dev(gK), dev(gV), dx, grads)
        torch.cuda.synchronize()
        assert ctx.device_wait_expired() == 0
        assert ctx.engine_name() == "backward"
        got_dx = dx.cpu().numpy().astype(np.float64)
        got = {k: v.cpu().numpy().astype(np.float64) for k, v in grads.items()}
    finally:
        ctx.rt_destroy()

    ref_dx, ref_dW, ref_dG = bwd.layer_backward(w, H, x, z.astype(np.float64), gy.astype(np.float64),
                                                None if gK is None else gK.astype(np.float64),
                                                None if gV is None else gV.astype(np.float64), gains=g, norm_free=norm_free, **kw)
    tol = tol or TOL[dtype]
    curve = rel_err_rows(got_dx, ref_dx).max(axis=0)
    errs = {"dx": curve.max()}
    for k in MATS:
        errs[k] = np.linalg.norm(got[k] - ref_dW[k]) / max(np.linalg.norm(ref_dW[k]), 1e-30)
    for k in GAINS:
        if norm_free:
            assert np.all(got[k] == 0.0), k
        elif ref_dG[k] is None:                        # RMS(z) sharing g_attn: its share is inside g_attn, g_kv is zero-filled
            assert k == "g_kv" and np.all(got[k] == 0.0)
        else:
            errs[k] = np.linalg.norm(got[k] - ref_dG[k]) / max(np.linalg.norm(ref_dG[k]), 1e-30)
    q = len(curve) // 4 or 1
    print("\n  [backward %s B=%d N=%d d=%d H=%d F=%d alibi=%g] dx by quarter of the sequence %s; %s" % (
        dtype, B, N, d, H, F, alibi, " ".join("%.1e" % curve[i:i + q].max() for i in range(0, len(curve), q)),
        " ".join("%s %.1e" % kv for kv in errs.items())))
    for k, e in errs.items():
        assert np.isfinite(e) and e <= tol, "%s: %.3e" % (k, e)


@pytest.mark.parametrize("B,N,d,H,F,alpha,scale,alibi,shared", [
    (2, 70, 128, 2, 256, 0.7, 0.5, 0.0, False),     # two tiles of Algorithm 1 run backwards (keys 0..31 and 32..63), ragged tail
    (1, 1, 128, 2, 512, 1.0, 1.0, 0.0, True),       # a single position: only the temporary pair
    (3, 33, 128, 2, 256, 1.0, 0.3, 8.0, True),      # one tile with a single query; bias; RMS(z) sharing g_attn
    (9, 40, 64, 1, 128, 0.5, 0.25, 0.0, False),     # more batch rows than one small-M launch takes
    (2, 200, 192, 3, 384, 0.6, 0.2, 8.0, False),    # tiles of 32, 64 and 128 keys; odd head count
])
def test_backward_fp32(oracle, B, N, d, H, F, alpha, scale, alibi, shared):
    _run(oracle, "f32", B, N, d, H, F, alpha=alpha, scale=scale, alibi=alibi, shared_kv_gain=shared)


def test_backward_fp32_norm_free(oracle):
    _run(oracle, "f32", 2, 45, 128, 2, 256, scale=0.02, norm_free=True)


def test_backward_fp32_without_pair_gradients(oracle):
    _run(oracle, "f32", 2, 50, 128, 2, 256, scale=0.5, with_pair_grads=False, gains="unit")


@pytest.mark.parametrize("B,N,d,H,F,scale,no_mfma", [(3, 200, 256, 4, 1024, 0.25, False), (8, 130, 512, 8, 2048, 0.125, False),
                                                     (2, 300, 1024, 16, 4096, 1.0, False),   # the headline width, unscaled logits
                                                     (2, 100, 768, 12, 3072, 0.25, False),   # three contraction steps per wavefront
                                                     (5, 333, 192, 3, 448, 0.25, False),     # ragged tiles of the products
                                                     (3, 200, 256, 4, 1024, 0.25, True)])    # fp32 products on bf16 storage
def test_backward_bf16_storage(oracle, B, N, d, H, F, scale, no_mfma):
    """bf16 storage: the batched products run on the matrix cores from bf16 copies of their operands (the recompute's
    activations as head + remainder), everything else in fp32; with RT_FLAG_NO_MFMA all of it is fp32."""
    _run(oracle, "bf16", B, N, d, H, F, scale=scale, alpha=0.7, no_mfma=no_mfma)


def test_backward_bf16_from_the_gpu_forward(oracle):
    """Forward on the GPU (rt_layer_prefill, bf16), backward from ITS output: the pipeline a training step runs.  The
    reference differentiates at the exact output, so the difference includes the forward's own error."""
    _run(oracle, "bf16", 4, 160, 256, 4, 1024, scale=0.125, alpha=0.7, z_from_gpu=True)


@pytest.mark.parametrize("kw", [
    dict(alibi=8.0, scale=0.3),                                   # positional bias in the matrix-core attention passes and the loop
    dict(norm_free=True, scale=0.02),                             # every normalisation the identity
    dict(shared_kv_gain=True, with_pair_grads=False, scale=0.5),  # RMS(z) sharing g_attn; no gradient arriving at K, V
])
def test_backward_bf16_variants(oracle, kw):
    """The single-launch reverse loop and the matrix-core attention passes (bf16 storage, d a multiple of 256) with the
    options the plain cases leave at their defaults; 170 positions: blocks of 32, 64 and 128 keys and a ragged last block."""
    _run(oracle, "bf16", 3, 170, 256, 4, 1024, alpha=0.8, **kw)


def test_backward_bf16_full_batch_headline_width(oracle):
    """B = 8 at d = 1024: the largest layout of the single-launch reverse loop (eight staged rows, 16 x 8 merge units)."""
    _run(oracle, "bf16", 8, 70, 1024, 16, 4096, scale=0.5, alpha=0.7)
