#!/usr/bin/env python3
"""Benchmark of the RT-layer prefill hot path on one MI355X.

A step is one rt_layer_prefill call (pre-pass, the N sequential base cases, every cross-block update)
on one batch of synthetic input already resident in HBM.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def measured_traffic(workload, what):
    """L2<->fabric bytes per launch from profiles/traffic.json: the rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs,
    already scaled by the copy-kernel calibration, each entry naming the commit it was measured on.  None if absent."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            ent = json.load(f)["%s/%s" % (workload, what)]
        return {"bytes": ent["bytes"], "measured_on": ent["commit"], "source": ent["source"]}
    except (OSError, KeyError, ValueError):
        return None


def method_bytes(B, N, d, H, F, E):
    """Bytes the METHOD has to move per layer call, by the per-token model of the tiled algorithm (Appendix C; footnote
    of Sec. 5 for the tile's reads): every level of Algorithm 1 reads q, k, v of a tile once and writes / reads each
    query's partial state once: 456 H ceil(log2 N) bytes per token at bf16; activations 11 d E per token (x twice,
    q / temporary pairs written and read, y, K, V written); the loop's five matrices and the three pre-pass matrices once
    (weights kept on chip)."""
    import math
    tokens = B * N
    # per level half of the positions are queries of a tile: q, k, v rows of one head read once and a partial state
    # (m, l, o[64], fp32) written once and read once = (3 * 64 E + 2 * 66 * 4) / 2 = 456 bytes per token and head at bf16
    per_level = (3 * 64 * E + 2 * 66 * 4) / 2.0
    return {"attention": float(per_level * H * math.ceil(math.log2(max(N, 2))) * tokens),
            "activations": 11.0 * d * E * tokens,
            "weights": float((11 + 3) * d * d * E) if F == 4 * d else float((3 * d * d + 2 * d * F + 3 * d * d) * E)}


def algorithmic_bytes(B, N, d, H, F, E, p_min, weights_resident):
    """Bytes one layer call must move (per-call totals), by term.

    weights      : the five matrices of the sequential loop (11 d^2 E bytes) are read once per call when the
                   engine keeps them on chip (persistent engine), once per position when they are streamed
                   (per-position engine); plus the three pre-pass matrices once.
    attention    : every cross-block event reads its q, k, v tiles once and writes a partial state that is
                   read once: (3*64*E + 2*66*4) bytes per (query, level, head, batch row), plus the direct
                   window rows.
    activations  : x read twice, Q / K_tmp / V_tmp written and read once, y / K / V written: 11 d E per token.
    """
    import math
    levels = 0
    attn = 0
    for t1 in range(1, N):
        P = t1 & -t1
        if P >= p_min:
            nq = min(P, N - t1)
            attn += B * H * (P * 2 * 64 * E + nq * 64 * E + 2 * nq * 66 * 4)
    window = sum((t & (p_min - 1)) for t in range(N)) * B * H * 2 * 64 * E
    return {
        "weights_seq": (1 if weights_resident else N) * (2 * d * d + 2 * d * F + d * d) * E * 1.0,
        "weights_pre": 3 * d * d * E * 1.0,
        "attention": float(attn + window),
        "activations": 11.0 * B * N * d * E,
    }


def stack_section(stream, layer_by_layer=True, reps=2, alibi=0.0, layers=0, positions=0):
    """The 12-layer stack workload (cfg5: B = 4, N = 4096) through the layer-wavefront engine (rt_stack_prefill: the
    layers run concurrently, a chunk of positions apart) and, for comparison, layer by layer (12 x rt_layer_prefill).
    Its bound is the weight stream: every (layer, position) reads the layer's five loop matrices once."""
    import numpy as np
    import torch
    from paper_2604_21215_amd import binding, inputs as gen, torch_io as tio
    from paper_2604_21215_amd.stack import DeviceStack
    ws = gen.WORKLOADS["cfg5"]
    if layers or positions:   # a reduced or enlarged variant of the workload (sweeps; not the benchmark line)
        import dataclasses
        ws = dataclasses.replace(ws, layers=layers or ws.layers, N=positions or ws.N)
    tabs = gen.make_embedding_tables(ws)
    sctx = binding.RTContext(ws.d, ws.H, ws.F, ws.B, ws.N, ws.dtype, resid_scale=ws.resid_scale, rms_eps=1e-6,
                             stream=stream.cuda_stream, alibi_max_bias=alibi)
    dls = [tio.DeviceLayer(gen.make_layer_weights(ws.seed, l, ws.d, ws.F, ws.dtype), None, ws.dtype)
           for l in range(ws.layers)]
    # table entries ~ N(0, 1): the scale at which the stack's parity tests run
    ds = DeviceStack(sctx, dls, gen.round_to_bf16(tabs["embedding"] * np.float32(50.0)), tabs["lm_head"], None, ws.dtype)
    ids = torch.from_numpy(np.ascontiguousarray(gen.make_token_ids(ws)[:, :ws.N], dtype=np.int32)).to("cuda:0")

    def timed(reps, **kw):
        ds.prefill(ids, ws.N, kv_cap=ws.N, **kw)   # warm-up (allocates the engine's scratch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ds.prefill(ids, ws.N, kv_cap=ws.N, **kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t_wf = timed(reps, wavefront=True)
    w_bytes = float(ws.N) * ws.layers * (3 * ws.d * ws.d + 2 * ws.d * ws.F) * 2
    sec = {
        "workload": "cfg5: %d RT layers, bf16, B=%d, N=%d, d_model=%d, embedding + read-out included"
                    % (ws.layers, ws.B, ws.N, ws.d),
        "us_per_step": t_wf * 1e6 / (ws.N + (ws.layers - 1) * 64),
        "ms_per_prefill": t_wf * 1e3, "tokens_per_s": ws.B * ws.N / t_wf,
        "layer_tokens_per_s": ws.B * ws.N * ws.layers / t_wf,
        "bound": "hbm", "algorithmic_bytes": w_bytes, "achieved": w_bytes / t_wf / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": w_bytes / t_wf / 1e9 / HBM_PEAK_GBS,
        "note": "algorithmic bytes = the loop matrices (3 d^2 + 2 d F elements) once per layer and position; "
                "host-timed over whole calls",
    }
    if layer_by_layer:
        t_seq = timed(1)
        sec["layer_by_layer_ms"] = t_seq * 1e3
        sec["speedup_over_layer_by_layer"] = t_seq / t_wf
    sctx.rt_destroy()
    return sec


def batch_sweep_section(stream, sizes=None):
    """rt_layer_prefill at the shapes of the paper's latency table (Sec. 6.2, Table 1: one layer, N = 512, d = 1024, 16 heads,
    batch sizes 32 .. 1024; bf16 here, logits scaled by 1/8): ms per call and what the paper measured on its own hardware.
    Context, not the headline: every batch size takes the engine rt_layer_prefill selects for it."""
    import numpy as np
    import torch
    from paper_2604_21215_amd import binding, inputs as gen, torch_io as tio
    d, H, F, N = 1024, 16, 4096, 512
    paper_ms = {32: 38.85, 64: 42.28, 128: 48.95, 256: 61.39, 512: 81.73, 1024: 134.09}
    li = gen.make_custom(3, "bf16", 32, N, d, H, F)
    dl = tio.DeviceLayer(li.weights, li.gains, "bf16")
    x32 = tio.to_device(li.x, "bf16")
    rows = []
    for B in (sizes or sorted(paper_ms)):
        x = x32.repeat(B // 32, 1, 1).contiguous()        # the same 32 sequences repeated: timing does not depend on the values
        y = torch.empty_like(x)
        K = torch.zeros((N, B, H, d // H), dtype=x.dtype, device=x.device)
        V = torch.zeros_like(K)
        ctx = binding.RTContext(d, H, F, B, N, "bf16", attn_scale=0.125, stream=stream.cuda_stream)
        try:
            ctx.rt_layer_prefill(dl.struct, x, y, K, V)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(2):
                ctx.rt_layer_prefill(dl.struct, x, y, K, V)
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 2
            rows.append({"B": B, "engine": ctx.engine_name(), "ms_per_call": ms, "us_per_position": ms * 1e3 / N,
                         "tokens_per_s": B * N / (ms * 1e-3), "paper_ms_other_hardware": paper_ms.get(B)})
        finally:
            ctx.rt_destroy()
        del x, y, K, V
    return {"workload": "one layer, N=512, d_model=1024, 16 heads, hidden 4096, bf16 (the shapes of the paper's Table 1)",
            "note": "paper_ms_other_hardware: the paper's figures with CUDA Graphs on one H100, quoted as context, not as a baseline",
            "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--engine", default="auto", choices=["auto", "stepwise", "graph", "persistent"])
    ap.add_argument("--p-min", type=int, default=0)
    ap.add_argument("--alibi", type=float, default=0.0,
                    help="maximum ALiBi bias (the paper's trained models: 8.0); 0 = the layer of Sec. 2.2 as it stands")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the rt_decode_step measurement")
    ap.add_argument("--no-parallel", action="store_true", help="skip rt_transformer_layer / rt_layer_recompute")
    ap.add_argument("--no-blocked", action="store_true",
                    help="skip rt_layer_prefill_blocked (thousands of launches: slow under a counter-collecting profiler)")
    ap.add_argument("--no-backward", action="store_true", help="skip rt_layer_backward")
    ap.add_argument("--no-stack", action="store_true", help="skip the 12-layer stack measurement (rt_stack_prefill)")
    ap.add_argument("--no-batch-sweep", action="store_true", help="skip rt_layer_prefill at N = 512 for batch sizes 32 .. 1024")
    ap.add_argument("--batch-sweep-only", action="store_true", help="only that sweep (for profiling): prints its section alone")
    ap.add_argument("--batch-sweep-sizes", default="", help="with --batch-sweep-only: comma-separated batch sizes, multiples of 32")
    ap.add_argument("--stack-only", action="store_true",
                    help="only the 12-layer stack through rt_stack_prefill (for profiling): prints its section alone")
    ap.add_argument("--stack-layers", type=int, default=0, help="with --stack-only: number of layers (default: the workload's 12)")
    ap.add_argument("--stack-positions", type=int, default=0, help="with --stack-only: sequence length (default: the workload's 4096)")
    ap.add_argument("--cpu-sample-positions", type=int, default=2048)
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy, the reference the rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "counters of the prefill kernel are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (one process, one device); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_21215_amd import binding, inputs as gen, torch_io as tio

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.traffic_calibration:
        big = torch.empty(256 * 2**20, dtype=torch.uint8, device="cuda:0")
        big.zero_()
        big2 = big.clone()          # one copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del big, big2
    if args.batch_sweep_only:
        sizes = [int(v) for v in args.batch_sweep_sizes.split(",") if v] or None
        print(json.dumps({"batch_sweep": batch_sweep_section(torch.cuda.current_stream(), sizes)}))
        return
    if args.stack_only:
        print(json.dumps({"stack_wavefront": stack_section(torch.cuda.current_stream(), layer_by_layer=False,
                                                           reps=args.steps, alibi=args.alibi, layers=args.stack_layers,
                                                           positions=args.stack_positions)}))
        return
    wl = gen.WORKLOADS[args.workload]
    li = gen.make_layer_inputs(wl)
    flags = {"auto": 0, "stepwise": binding.RT_FLAG_ENGINE_STEPWISE,
             "graph": binding.RT_FLAG_ENGINE_STEPWISE | binding.RT_FLAG_HIP_GRAPH,
             "persistent": binding.RT_FLAG_ENGINE_PERSISTENT}[args.engine]
    stream = torch.cuda.current_stream()
    ctx = binding.RTContext(wl.d, wl.H, wl.F, wl.B, wl.N, wl.dtype, p_min=args.p_min, resid_scale=wl.resid_scale,
                            attn_scale=1.0, rms_eps=1e-6, flags=flags, stream=stream.cuda_stream, alibi_max_bias=args.alibi)
    dl = tio.DeviceLayer(li.weights, li.gains, wl.dtype)
    xd = tio.to_device(li.x, wl.dtype)
    y = torch.empty_like(xd)
    K = torch.zeros((wl.N, wl.B, wl.H, wl.head_dim), dtype=xd.dtype, device=xd.device)
    V = torch.zeros_like(K)

    for _ in range(args.warmup):
        ctx.rt_layer_prefill(dl.struct, xd, y, K, V)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record(stream)
    for i in range(args.steps):
        ctx.rt_layer_prefill(dl.struct, xd, y, K, V)
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert ctx.device_wait_expired() == 0, "a device-side wait expired: results invalid"
    per_call_ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    ms_per_step = wall * 1e3 / args.steps
    tokens = wl.B * wl.N
    value = tokens * args.steps / wall
    engine = ctx.engine_name()

    E = 2 if wl.dtype == "bf16" else 4
    p_min = ctx.cfg.p_min if ctx.cfg.p_min else 32
    resident = engine == "persistent"
    terms = algorithmic_bytes(wl.B, wl.N, wl.d, wl.H, wl.F, E, p_min, resident)
    streamed = algorithmic_bytes(wl.B, wl.N, wl.d, wl.H, wl.F, E, p_min, False)
    design_bytes = sum(terms.values())
    mterms = method_bytes(wl.B, wl.N, wl.d, wl.H, wl.F, E)
    alg_bytes = sum(mterms.values()) if resident else design_bytes
    dev_ms = float(np.mean(per_call_ms))
    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    traffic = measured_traffic(args.workload, engine)
    roofline = {
        "bound": "hbm",
        "kernel": ("persistent_kernel (one launch per call; the call's two small pre-pass kernels are inside the timed events)"
                   if resident else "rt_layer_prefill (%s engine, all launches of one call)" % engine),
        "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
        "traffic": traffic["bytes"] if traffic else None, "traffic_source": traffic,
        "traffic_over_algorithmic": (traffic["bytes"] / alg_bytes) if traffic else None,
        "launch_ms": dev_ms, "algorithmic_bytes": alg_bytes, "algorithmic_terms": mterms if resident else terms,
        # the same count with this build's own choices added (blocks below p_min read directly by each query: the window)
        "design_bytes": design_bytes, "design_terms": terms,
        "us_per_position": dev_ms * 1e3 / wl.N,
        # what a design that re-streams the loop's weights at every position would have to move, for comparison
        "weight_streaming_equivalent_GBps": sum(streamed.values()) / (dev_ms * 1e-3) / 1e9,
    }
    attn_flops = 2.0 * wl.N * (wl.N - 1) * wl.d * wl.B
    out = {
        "metric": "RT-layer prefill tokens/s at N=2048,d=1024 (1 GPU)" if args.workload == "cfg3"
        else "RT-layer prefill tokens/s (%s)" % args.workload,
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: single RT layer, %s, B=%d, N=%d, d_model=%d, %d heads x 64, MLP hidden %d"
                   % (wl.name, wl.dtype, wl.B, wl.N, wl.d, wl.H, wl.F), "engine": engine, "p_min": p_min,
                   "alibi_max_bias": args.alibi,
                   "attention_gflop_per_call": attn_flops / 1e9},
        "roofline": roofline,
    }

    # The cross-block UpdateTile kernel by itself (the path's one dense contraction): the top three levels carry
    # 87.5 % of the attention FLOPs of a call; each event is re-run alone on the state the last call left.
    if wl.dtype == "bf16" and wl.N >= 256:
        levels = []
        for lv in range(3):
            P = wl.N >> (lv + 1)
            evs = [(t1, min(P, wl.N - t1)) for t1 in range(P, wl.N, 2 * P)]
            if P < 64 or not evs:
                continue
            reps = 10
            for t1, nq in evs:
                ctx.rt_cross_block_event(K, V, t1, P, nq)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                for t1, nq in evs:
                    ctx.rt_cross_block_event(K, V, t1, P, nq)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (reps * len(evs))
            fl = float(np.mean([4.0 * P * nq * wl.head_dim * wl.B * wl.H for _, nq in evs]))
            levels.append({"P": P, "events_per_call": len(evs), "us_per_event": us, "tflops": fl / us / 1e6})
        if levels:
            tot_fl = sum(l["tflops"] * l["us_per_event"] * l["events_per_call"] for l in levels)
            tot_us = sum(l["us_per_event"] * l["events_per_call"] for l in levels)
            hp = engine == "persistent"   # the tile then takes fp16 copies of the unrounded queries and keys
            out["cross_block_kernel"] = {
                "bound": "mfma", "unit": "TFLOP/s", "peak": MFMA_BF16_PEAK_TFLOPS * 1e0,
                "achieved": tot_fl / tot_us, "frac": tot_fl / tot_us / MFMA_BF16_PEAK_TFLOPS,
                "logits": "one fp16 product from unrounded queries and keys" if hp else "bf16",
                "note": "stand-alone launches of the top three levels (87.5 % of the attention FLOPs), FLOP-weighted, in the "
                        "form the engine of the timed call uses; achieved counts the algorithmic 4 P nq 64 FLOPs per "
                        "(b, h) event = what the matrix pipeline executes; back-to-back launches, launch overhead included",
                "levels": levels}

    # One decoding step (rt_decode_step) over the cache the call above left: position t = N - 1 is evaluated again
    # from rows 0 .. N-2 (row N-1 is rewritten with the same values).  Bandwidth-bound in principle: the step has to
    # read the cache (2 t B d E bytes) and the layer's weights (12 d^2 E) once.
    if not args.no_decode:
        t_dec = wl.N - 1
        x_t = xd[:, t_dec].contiguous()
        y_t = torch.empty_like(x_t)
        for _ in range(3):
            ctx.rt_decode_step(dl.struct, x_t, t_dec, y_t, K, V)
        reps = 50
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            ctx.rt_decode_step(dl.struct, x_t, t_dec, y_t, K, V)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        dec_bytes = 2.0 * t_dec * wl.B * wl.d * E + 12.0 * wl.d * wl.d * E
        out["decode_step"] = {"t": t_dec, "us_per_step": us, "tokens_per_s": wl.B / (us * 1e-6), "bound": "hbm",
                              "algorithmic_bytes": dec_bytes, "achieved": dec_bytes / (us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": dec_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                              "traffic": (measured_traffic(args.workload, "decode" if ctx.engine_name() == "decode-single-launch"
                                                            else "decode_multi_launch") or {}).get("bytes") if t_dec == 2047 else None,
                              "engine": ctx.engine_name(),
                              "note": "one launch per step (256 workgroups, weight slices in LDS, cache rows and matrices requested at "
                                      "its start)" if ctx.engine_name() == "decode-single-launch" else
                                      "eight launches per step on one stream (bf16: products on the matrix cores)"}

    # The same layer without its sequential loop (every key-value pair known in advance): the recompute from a given
    # output (Sec. 6.1) and the standard Transformer layer (Sec. 2.1) - the paper's Figure 4 compares the tiled RT layer
    # with the latter.  GEMM-bound: 2 M (d^2 + 2 d F) FLOPs of the block + 2 M 3 d^2 per pre-pass + the attention.
    if wl.dtype == "bf16" and not args.no_parallel:
        y2, K2, V2 = torch.empty_like(y), torch.zeros_like(K), torch.zeros_like(V)
        Mrows = wl.B * wl.N
        blk = 2.0 * Mrows * (wl.d * wl.d + 2.0 * wl.d * wl.F)
        pre = 2.0 * Mrows * 3.0 * wl.d * wl.d
        sec = {}
        for name, fn, fl in (("transformer_layer", lambda: ctx.rt_transformer_layer(dl.struct, xd, y2, K2, V2), blk + pre + attn_flops),
                             ("recompute", lambda: ctx.rt_layer_recompute(dl.struct, xd, y, y2, K2, V2), blk + 2 * pre + attn_flops)):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 5
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            sec[name] = {"ms_per_call": ms, "tokens_per_s": tokens / (ms * 1e-3), "gflop": fl / 1e9, "bound": "mfma",
                         "achieved": fl / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        # blocked recurrence (Sec. 8): the sequential loop over blocks of S positions, S x B rows per matrix product
        blocked = {}
        for S in (() if args.no_blocked else (4, 16, 32)):
            fnb = lambda: ctx.rt_layer_prefill_blocked(dl.struct, xd, S, y2, K2, V2)
            fnb()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(2):
                fnb()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 2
            blocked["block_%d" % S] = {"ms_per_call": ms, "tokens_per_s": tokens / (ms * 1e-3)}
        if blocked:
            sec["blocked_recurrence"] = blocked
        sec["rt_layer_prefill_ms"] = dev_ms
        sec["rt_over_transformer"] = dev_ms / sec["transformer_layer"]["ms_per_call"]
        out["loop_free_layers"] = sec

    # Backward pass of the same layer (Sec. 6.4) from the output the timed calls left in y: recompute from (x, z), the
    # reverse loop over positions (it carries the gradients of the persistent pairs only), batched parameter sums.
    if not args.no_backward:
        gen_t = torch.Generator(device="cuda:0")
        gen_t.manual_seed(wl.seed)
        gy = torch.randn(xd.shape, generator=gen_t, device="cuda:0", dtype=torch.float32).to(xd.dtype)
        dx = torch.empty(xd.shape, dtype=torch.float32, device="cuda:0")
        grads = {k: torch.empty(tuple(li.weights[k].shape), dtype=torch.float32, device="cuda:0")
                 for k in ("Wq", "Wk", "Wv", "Wo", "W1", "W2")}
        ctx.rt_layer_backward(dl.struct, xd, y, gy, None, None, dx, grads)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 2
        e0.record(stream)
        for _ in range(reps):
            ctx.rt_layer_backward(dl.struct, xd, y, gy, None, None, dx, grads)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out["backward"] = {"ms_per_call": ms, "tokens_per_s": tokens / (ms * 1e-3), "us_per_position": ms * 1e3 / wl.N,
                           "over_forward": ms / dev_ms, "dtype": "f32 arithmetic, %s storage" % wl.dtype,
                           "finite": bool(torch.isfinite(dx).all().item())}
        del gy, dx, grads

    if not args.no_cpu_baseline:
        from oracle import rt_oracle
        n_s = min(args.cpu_sample_positions, wl.N)
        w64 = {k: v.astype(np.float64) for k, v in li.weights.items()}
        lay = rt_oracle.Layer(w64, wl.H, alpha=wl.resid_scale, eps=1e-6, alibi_max_bias=args.alibi)
        xs = li.x[:, :n_s].astype(np.float64)
        t0 = time.perf_counter()
        ref = lay.prefill(xs)
        dt = time.perf_counter() - t0
        cores = min(rt_oracle.max_threads(), wl.B) if wl.B >= 4 else rt_oracle.max_threads()
        out["cpu_baseline"] = {"value": wl.B * n_s / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": "first %d positions of all %d sequences of the same workload (%.1f s)"
                               % (n_s, wl.B, dt)}
        got = tio.to_host(y[:, :n_s])
        err = (np.linalg.norm(got - ref[0], axis=-1) / np.linalg.norm(ref[0], axis=-1)).max(axis=0)
        br_ref, br_got = ref[0] - xs, got - xs     # the attention + MLP branch alone (y = x + branch hides its error)
        ebr = (np.linalg.norm(br_got - br_ref, axis=-1) / np.linalg.norm(br_ref, axis=-1)).max(axis=0)
        gK, gV = tio.to_host(K[:n_s]), tio.to_host(V[:n_s])
        eK = (np.linalg.norm(gK - ref[1][:n_s], axis=-1) / np.linalg.norm(ref[1][:n_s], axis=-1)).reshape(n_s, -1).max(axis=1)
        eV = (np.linalg.norm(gV - ref[2][:n_s], axis=-1) / np.linalg.norm(ref[2][:n_s], axis=-1)).reshape(n_s, -1).max(axis=1)
        qs = [slice(i * n_s // 4, max((i + 1) * n_s // 4, i * n_s // 4 + 1)) for i in range(4)]
        out["parity_sample"] = {"max_rel_err_y": float(err.max()), "max_rel_err_K": float(eK.max()),
                                "max_rel_err_V": float(eV.max()), "max_rel_err_branch": float(ebr.max()),
                                "by_quarter_of_the_sequence": {"y": [float(err[q].max()) for q in qs],
                                                               "K": [float(eK[q].max()) for q in qs],
                                                               "V": [float(eV[q].max()) for q in qs],
                                                               "branch": [float(ebr[q].max()) for q in qs]},
                                "positions": n_s, "tolerance": 2e-2 if wl.dtype == "bf16" else 1e-4}
    ctx.rt_destroy()

    if not args.no_stack and args.workload == "cfg3":
        out["stack_wavefront"] = stack_section(stream, alibi=args.alibi)
    if not args.no_batch_sweep and args.workload == "cfg3":
        try:
            out["batch_sweep"] = batch_sweep_section(stream)
        except Exception as exc:   # context only: never lose the headline line over it
            out["batch_sweep"] = {"error": repr(exc)[:300]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
