"""Writes the sampled oracle rows under tests/golden/ that the GPU parity tests of the long workloads compare
against -- TEST INFRASTRUCTURE ONLY.

The fp64 oracle needs minutes at these sizes (sequence lengths 4096 and 8192 of the sequence-length sweep; the
12-layer stack at 4096 positions plus 128 decoding steps), so it is run once, here, on the CPU, and a sample of
its output rows is stored as float32.  Every stored value comes from oracle/rt_oracle.py alone, fed by the seeded
input generator (paper_2604_21215_amd/inputs.py: draws and storage rounding only); nothing in this script imports,
loads or calls the HIP library.

    python -m oracle.write_golden sweep        -> tests/golden/oracle_rows_sweep_b2_n8192.npz
    python -m oracle.write_golden stack_unit   -> tests/golden/oracle_rows_stack_unit_table.npz
    python -m oracle.write_golden stack_literal-> tests/golden/oracle_rows_stack_literal_table.npz

sweep: one RT layer (Sec. 2.2), bf16-rounded inputs, B = 2, d = 1024, 16 heads, hidden 4096, one run at N = 8192.
    Position t of the layer depends on positions <= t only (the layer is causal), and the sweep's shorter inputs are
    prefixes of the longest, so the rows below 4096 also are the references of the N = 4096 run.
stack_unit / stack_literal: 12 stacked RT layers (alpha = 1/sqrt(12)), B = 4, token ids uniform over 32768, untied
    read-out after a final RMS; the oracle runs all 4096 + 128 positions as ONE prefill -- a decoding step is the same
    recurrence continued (Sec. 7.3; pinned on the CPU: prefill(N) = prefill(N - k) + k decoding steps), so rows
    4096.. are the references of the decoding steps.
      stack_unit:    embedding table multiplied by 50 (entries ~ N(0, 1)), logits unscaled (attn_scale 1)
      stack_literal: embedding table as drawn (entries ~ N(0, 0.02^2)), attn_scale 1/8
    (the literal table with unscaled logits is ill-conditioned: a CPU pin shows the oracle itself moving by far more
    than the tolerance under a perturbation of one storage rounding, so no stored rows could be met there.)

Stored per file: `positions_y`, `positions_kv` (0-based), `y` [L, P, B, d], `K`, `V` [L, Pkv, B, H, 64], for the
stacks `positions_logits`, `logit_columns` and `logits` [Plog, B, columns] (a fixed subsample of the vocabulary),
and `fingerprint` (sums over the generated inputs: a test that regenerates other inputs must not use the file).
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if _ROOT not in sys.path:
    sys.path.insert(0, _ROOT)

from oracle import rt_oracle  # noqa: E402
from paper_2604_21215_amd import inputs as gen  # noqa: E402

GOLDEN = os.path.join(_ROOT, "tests", "golden")

SWEEP_POSITIONS = [0, 1, 31, 32, 33, 255, 256, 1023, 1024, 2047, 2048, 2049, 2050, 2081, 3071, 3072, 3583, 4094, 4095,
                   4096, 4097, 4098, 4129, 5000, 5119, 5120, 6143, 6144, 6145, 7167, 7679, 8000, 8190, 8191]

STACK_SAMPLES = {
    # name: (embedding multiplier, attn_scale, positions of y, positions of K and V, positions of the logits)
    "stack_unit": (50.0, 1.0,
                   [0, 255, 511, 512, 513, 1023, 1024, 1025, 2047, 2048, 2049, 3071, 3072, 4000, 4094, 4095, 4096, 4160, 4223],
                   [512, 2049, 4095, 4096, 4223], [4095, 4096, 4160, 4223]),
    "stack_literal": (1.0, 0.125,
                      [0, 511, 512, 1024, 2048, 2049, 3072, 4095, 4096, 4160, 4223],
                      [2049, 4095, 4223], [4095, 4096, 4223]),
}
LOGIT_STRIDE = 16   # every 16th vocabulary entry


def _layer(weights, H, **kw):
    return rt_oracle.Layer({k: v.astype(np.float64) for k, v in weights.items()}, H, **kw)


def write_sweep():
    wl = gen.WORKLOADS["cfg4_8192"]
    li = gen.make_layer_inputs(wl)
    x = li.x.astype(np.float64)
    t0 = time.time()
    y, K, V = _layer(li.weights, wl.H, alpha=wl.resid_scale, eps=1e-6).prefill(x)
    print("sweep: oracle over %d x %d positions in %.0f s" % (wl.B, wl.N, time.time() - t0), flush=True)
    pos = np.array(SWEEP_POSITIONS, dtype=np.int32)
    out = os.path.join(GOLDEN, "oracle_rows_sweep_b2_n8192.npz")
    np.savez_compressed(out, positions_y=pos, positions_kv=pos,
                        y=y[:, pos].transpose(1, 0, 2)[None].astype(np.float32),
                        K=K[pos][None].astype(np.float32), V=V[pos][None].astype(np.float32),
                        fingerprint=np.array([x.sum(), np.abs(x).sum(), li.weights["W2"].astype(np.float64).sum()]))
    print("wrote", out, os.path.getsize(out), "bytes", flush=True)


def write_stack(name):
    mult, attn_scale, pos_y, pos_kv, pos_lg = STACK_SAMPLES[name]
    wl = gen.WORKLOADS["cfg5"]
    T = wl.N + wl.decode_steps
    ids = gen.make_token_ids(wl)
    tabs = gen.make_embedding_tables(wl)
    emb = tabs["embedding"]
    if mult != 1.0:
        emb = gen.round_to_bf16(emb * np.float32(mult))
    x = rt_oracle.embed(emb.astype(np.float64), ids[:, :T])
    pos_y, pos_kv, pos_lg = (np.array(p, dtype=np.int32) for p in (pos_y, pos_kv, pos_lg))
    ys, Ks, Vs = [], [], []
    t0 = time.time()
    for l in range(wl.layers):
        w = gen.make_layer_weights(wl.seed, l, wl.d, wl.F, wl.dtype)
        y, K, V = _layer(w, wl.H, alpha=wl.resid_scale, eps=1e-6, attn_scale=attn_scale).prefill(x)
        ys.append(y[:, pos_y].transpose(1, 0, 2).astype(np.float32))
        Ks.append(K[pos_kv].astype(np.float32))
        Vs.append(V[pos_kv].astype(np.float32))
        x = y
        print("%s: layer %d done, %.0f s" % (name, l, time.time() - t0), flush=True)
    cols = np.arange(0, wl.vocab, LOGIT_STRIDE, dtype=np.int32)
    W_lm = tabs["lm_head"].astype(np.float64)[cols]
    logits = np.stack([rt_oracle.lm_head(W_lm, x[:, p], None, 1e-6) for p in pos_lg]).astype(np.float32)
    out = os.path.join(GOLDEN, "oracle_rows_%s_table.npz" % name)
    np.savez_compressed(out, positions_y=pos_y, positions_kv=pos_kv, positions_logits=pos_lg, logit_columns=cols,
                        y=np.stack(ys), K=np.stack(Ks), V=np.stack(Vs), logits=logits,
                        embedding_multiplier=np.array(mult), attn_scale=np.array(attn_scale),
                        fingerprint=np.array([float(ids.sum()), emb.astype(np.float64).sum(),
                                              np.abs(emb.astype(np.float64)).sum()]))
    print("wrote", out, os.path.getsize(out), "bytes", flush=True)


def main(argv):
    os.makedirs(GOLDEN, exist_ok=True)
    rt_oracle.build()
    for what in (argv or ["sweep", "stack_unit", "stack_literal"]):
        if what == "sweep":
            write_sweep()
        elif what in STACK_SAMPLES:
            write_stack(what)
        else:
            raise SystemExit("unknown sample %r" % what)


if __name__ == "__main__":
    main(sys.argv[1:])
