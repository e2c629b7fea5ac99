#!/usr/bin/env python3
"""Throughput of the Ladder-Residual shard forward on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 70b_r8_decode] [--mode decode|prefill]

mode decode (default): a step = one decode step of the whole block stack (all 2N modules: RMSNorm, QKV,
rotary + cache append, split-KV attention, O projection, SwiGLU MLP, partial-sum reduce + residual add)
for one batch, in the fused schedule (161 launches for 80 layers).  Workload 70b_r8_decode: 80 layers of
a 70B-shaped TP rank at R = 8 (hidden 8192, 8 q / 1 kv heads, d = 128, intermediate 3584), batch 4,
synthetic KV cache of 1024 positions, 7 synthetic peer partial sums per module.  All inputs are seeded,
synthetic and resident in HBM before the timed region.
mode prefill: a step = one prefill call (workload 70b_r4_prefill: 16 x 2048 tokens).

With no --mode the default run is the whole metric: the decode workload (REPS timed regions of K steps each,
every region over the same cache positions; the median is reported), then, on a fresh context, the prefill
workload 70b_r4_prefill (median of 3 calls), reported under "prefill" in the same line.

Prints ONE JSON line: the contract fields plus "roofline" (dominant kernel: HIP events attached to every
dispatch in an instrumented pass right after the timed one; "traffic" = HBM bytes per launch counted by
rocprofv3, read from the committed summary under profiles/, with its source) and "cpu_baseline" (the CPU
oracle timed on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def build_context(w, device, extra_seq, peers_rows, layer0=0, **override):
    """A context with the workload's layers layer0 .. layer0 + w.n_layers - 1 (layer0 > 0: a later pipeline stage)."""
    import torch
    from paper_2501_06589_amd import inputs, ladder
    cfg = ladder.config_for(w, max_seq=w.prefill + w.kv_preload + extra_seq, **override)
    ctx = ladder.Ladder(cfg)
    t0 = time.time()
    for i in range(w.n_layers):
        for r in range(w.n_real_shards):
            ctx.load_layer(i, r, inputs.layer_weights(w, layer0 + i, r, device))
        if i % 16 == 15:
            torch.cuda.synchronize()
            log(f"[bench] weights: {i + 1}/{w.n_layers} layers generated and packed ({time.time() - t0:.1f}s)")
    peers = inputs.peer_partials(w, peers_rows, device) if w.n_peers else None
    if peers is not None:
        ctx.set_peer_partials(peers)
    torch.cuda.synchronize()
    return ctx


def read_profile_value(path, key):
    """'<key>: <number>' line of a committed profile summary, or None."""
    import re
    if not os.path.exists(path):
        return None
    m = re.search(r"^" + re.escape(key) + r":\s*([0-9.eE+-]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def decode_algorithmic_bytes(w, s_mean):
    """Bytes one decode step must move: every weight once, the visible KV cache once, peers once."""
    weights = w.n_layers * w.n_real_shards * w.params_per_layer() * 2
    kv = w.n_layers * w.n_real_shards * w.batch * w.n_kv_heads * w.head_dim * 2 * 2 * s_mean
    peers = 2 * w.n_layers * w.n_peers * w.batch * w.hidden * 2
    return weights, kv, peers


def cpu_baseline_decode(w, device, n_layers_sample, kv_len):
    """The oracle as it stands, one decode step on the first n_layers_sample layers of the workload."""
    import numpy as np
    import torch
    from oracle import from_torch
    from oracle import ladder_oracle as lo
    from paper_2501_06589_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    ws = w.with_(n_layers=n_layers_sample)
    cfg = from_torch.config_from_workload(ws)
    layers = [from_torch.layer_from_tensors([{k: v.cpu() for k, v in inputs.layer_weights(ws, i, r, device).items()}
                                             for r in range(ws.n_real_shards)]) for i in range(n_layers_sample)]
    n_steps = 20   # about 10 s of CPU work on the box's 16 host cores
    state = lo.State.empty(cfg, ws.n_real_shards, ws.batch, kv_len + n_steps + 1)
    for i in range(n_layers_sample):
        for r in range(ws.n_real_shards):
            k, v = inputs.kv_cache(ws, i, r, ws.batch, kv_len, device)
            from_torch.load_kv(state, i, r, k, v)
    state.pos = kv_len
    peers = inputs.peer_partials(ws, ws.batch, device)
    opeers = from_torch.to_f64(peers) if peers is not None else None
    e = from_torch.to_f64(inputs.embeddings(ws, ws.batch, 1, inputs.SEED_DECODE0, device))
    t0 = time.perf_counter()
    for i in range(n_steps):
        if i:
            e = from_torch.to_f64(inputs.embeddings(ws, ws.batch, 1, inputs.SEED_DECODE0 + i, device))
        lo.forward_eq2(e, layers, cfg, state, opeers)
    dt = (time.perf_counter() - t0) / n_steps
    full_step_s = dt * w.n_layers / n_layers_sample
    return {"value": w.batch / full_step_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_steps} decode steps (batch {w.batch}, {kv_len}+ cached positions) of the first {n_layers_sample} "
                      f"of {w.n_layers} layers, {dt:.2f} s per step, scaled linearly to {w.n_layers} layers"}


def run_decode(args):
    import torch
    from paper_2501_06589_amd import inputs, ladder
    w = inputs.WORKLOADS[args.workload]
    if args.layers:
        w = w.with_(n_layers=args.layers)
    if args.batch:
        w = w.with_(batch=args.batch)
    if args.kv and w.kv_preload:
        w = w.with_(kv_preload=args.kv)
    if args.no_peers:
        w = w.with_(tp_degree=w.n_real_shards)
    dev = "cuda:0"
    prof_steps = 8
    total_steps = args.warmup + args.steps + prof_steps
    reps = max(1, args.reps)
    # the peer tensor must hold as many rows per set as the configuration announces (peer_rows)
    ctx = build_context(w, dev, total_steps + (3 if args.timeline else 0), w.batch * max(w.prefill, 1), max_tokens=max(w.prefill, 1),
                        decode_graph=1 if args.graph else 0, overlap_modules=0 if args.no_overlap else 1,
                        decode_fused=0 if args.no_fused else {"paired": 1, "single": 2, "chain": 3}[args.fused_plan],
                        reduce_delay_us=args.reduce_delay_us, n_standard_layers=args.standard_layers,
                        wiring={"ladder": ladder.LADDER_WIRING_LADDER, "standard": ladder.LADDER_WIRING_STANDARD,
                                "parallel": ladder.LADDER_WIRING_PARALLEL}[args.wiring])
    # the cache as it stands before the first decode step: a synthetic one (kept, so that every timed region can
    # start from the same positions) or the one a prefill leaves
    kv = [[inputs.kv_cache(w, i, r, w.batch, w.kv_preload, dev) for r in range(w.n_real_shards)]
          for i in range(w.n_layers)] if w.kv_preload else None
    emb_prefill = None if w.kv_preload else inputs.embeddings(w, w.batch, w.prefill, inputs.SEED_PREFILL, dev)

    def reset_cache():
        if kv is not None:
            for i in range(w.n_layers):
                for r in range(w.n_real_shards):
                    ctx.load_kv(i, r, kv[i][r][0], kv[i][r][1])
        else:
            ctx.prefill(emb_prefill)

    reset_cache()
    xs = torch.stack([inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0 + i, dev)[:, 0] for i in range(total_steps)])
    out = torch.empty((w.batch, w.hidden), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] context ready: {ctx.device_bytes() / 2**30:.2f} GiB on device")
    copy_gbps = None
    if args.copy_calibration or not args.no_ceiling:
        # plain copy kernel, 1 GiB read + 1 GiB written per launch: the known-size dispatch that scales rocprofv3's
        # FETCH_SIZE / WRITE_SIZE counters, and a measured ceiling for streaming kernels on this machine
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        ctx.calibration_copy(dst, src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(4):
            ctx.calibration_copy(dst, src)
        torch.cuda.synchronize()
        copy_gbps = 4 * 2 * src.numel() * 4 / (time.perf_counter() - t0) / 1e9
        del src, dst
    head_vocab, toks = None, None
    if args.head:
        vocab = 128256 if w.hidden >= 4096 else 32000          # Llama-3 / Llama-2 vocabulary sizes
        head_vocab = (vocab, vocab // w.tp_degree)
        hw = inputs.head_weights(w, vocab, vocab // w.tp_degree, device=dev)
        ctx.load_head(hw["table"], hw["final_norm"], hw["w_lm"])
        toks = inputs.prompt_tokens(w.batch, 1, vocab, dev)[:, 0].contiguous()
        del hw

    def step(i):
        nonlocal toks
        if args.head:
            ctx.decode_step(ctx.embed(toks), out)
            toks = ctx.head(out, want_logits=False)[1]
        else:
            ctx.decode_step(xs[i], out)

    # reps timed regions of exactly K steps, each after W untimed warm-up steps from the same cache state
    rep_ms = []
    pos_start = pos_end = 0
    for rep in range(reps):
        if rep:
            reset_cache()
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        pos_start = ctx.position()[0]
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        rep_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)
        pos_end = ctx.position()[0]
        assert torch.isfinite(out).all()
    ms_per_step = sorted(rep_ms)[len(rep_ms) // 2]      # the median region
    tokens_per_s = w.batch / (ms_per_step * 1e-3)
    s_mean = (pos_start + pos_end + 1) / 2.0           # visible positions averaged over the timed steps
    wb, kvb, pb = decode_algorithmic_bytes(w, s_mean)
    step_bytes = wb + kvb + pb

    # instrumented pass: HIP events around every launch, on the stream it is launched on
    ctx.profile_enable(True)
    ctx.profile_reset()
    for i in range(prof_steps):
        ctx.decode_step(xs[args.warmup + args.steps + i], out)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    fused = bool(prof.get("fused_decode", (0, 0.0))[0])
    if fused:
        # fused path: every launch is the same kernel (one or two projections and/or the attention of
        # one layer); algorithmic bytes of a step (weights + visible KV + peers) over its launches
        n_gemv, ms_gemv = prof["fused_decode"]
        chained = n_gemv == prof_steps     # one launch per step: the chained step
        kernel_name = ("fused_chain_kernel (a whole decode step: persistent workgroups run the step's weight-streaming skinny "
                       "GEMM jobs and split-KV attention jobs, which meet at completion flags)" if chained else
                       "fused_decode_kernel (decode: weight-streaming skinny GEMM jobs + split-KV attention job)")
        gemv_bytes_per_launch = step_bytes / (n_gemv / prof_steps)
    else:
        chained = False
        kernel_name = "gemv_mfma_kernel (decode weight-streaming skinny GEMM)"
        n_gemv, ms_gemv = prof["gemv"]
        gemv_bytes_per_launch = wb / (4 * w.n_layers * w.n_real_shards)   # 4 projections per layer and shard
    avg_ms = ms_gemv / max(n_gemv, 1)
    achieved = gemv_bytes_per_launch / (avg_ms * 1e-3) / 1e9 if n_gemv else 0.0
    kname = ("fused_chain" if chained else "fused_decode") if fused else "gemv"
    traffic_file = os.path.join("profiles", f"{kname}_hbm_traffic_{w.name}.md")
    traffic = read_profile_value(os.path.join(ROOT, traffic_file), "traffic_bytes_per_launch")
    trace_file = os.path.join("profiles", f"{kname}_kernel_{w.name}.md")
    prof_avg_us = read_profile_value(os.path.join(ROOT, trace_file), "rocprofv3_avg_launch_us")
    roofline = {"bound": "hbm", "kernel": kernel_name,
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_source": traffic_file if traffic else None,
                "algorithmic_bytes_per_launch": gemv_bytes_per_launch,
                "avg_launch_ms": avg_ms, "launches": n_gemv,
                "duration_source": f"HIP events attached to every dispatch of {prof_steps} steps after the timed regions, "
                                   "on the stream the kernel is launched on" +
                                   ("" if chained else "; excludes the ~1.5 us between launches"),
                # the same figures from the committed rocprofv3 kernel trace (a separate run of this command)
                "rocprofv3": ({"avg_launch_us": prof_avg_us, "frac": gemv_bytes_per_launch / (prof_avg_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                               "source": trace_file} if prof_avg_us else None),
                # algorithmic bytes of a step over the measured step time, launch gaps included
                "frac_whole_step": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS}
    per_class = {k: {"launches": n, "avg_us": (ms / n * 1e3 if n else 0.0), "ms_per_step": ms / prof_steps}
                 for k, (n, ms) in prof.items() if n}
    timeline = chain_timeline(ctx, xs[args.warmup], out) if (args.timeline and chained) else None
    ctx.free()
    del ctx, kv
    torch.cuda.empty_cache()
    cpu = cpu_baseline_decode(w, dev, min(args.cpu_layers, w.n_layers), w.kv_preload or w.prefill) if not args.no_cpu else None
    whole_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    return {
        "metric": "decode_tokens_per_s", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "repetitions": {"n": reps, "ms_per_step": rep_ms, "reported": "median"},
        "config": {"workload": w.name, "n_layers": w.n_layers, "hidden": w.hidden, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "inter": w.inter, "tp_degree": w.tp_degree,
                   "batch": w.batch, "kv_positions": [pos_start, pos_end], "peers": w.n_peers,
                   **({"head_vocab": head_vocab[0], "head_vocab_local": head_vocab[1]} if head_vocab else {})},
        "hbm": {"algorithmic_bytes_per_step": step_bytes, "weights": wb, "kv": kvb, "peers": pb,
                "achieved_GBps_whole_step": whole_gbps,
                "frac_of_peak_whole_step": whole_gbps / HBM_PEAK_GBS,
                "measured_copy_GBps": copy_gbps,
                "frac_of_measured_copy_whole_step": (whole_gbps / copy_gbps) if copy_gbps else None},
        "roofline": roofline, "kernel_classes": per_class, "cpu_baseline": cpu,
        **({"timeline": timeline} if timeline else {}),
    }


def chain_timeline(ctx, x, out):
    """Inside a chained decode step (one launch, so events around it say nothing about its parts): the library's
    timeline of one step, reduced to the steady state of the middle layers.  Per kind of job the time from its first
    block's inputs being complete to its last block's end, the distance between consecutive layers, and the two phases
    of a ladder layer: {attention -> o || gate/up} and {qkv || down}.  Microseconds."""
    import numpy as np
    for _ in range(2):
        ctx.decode_step(x, out)
    ctx.timeline_enable(True)
    ctx.decode_step(x, out)
    rec, rate = ctx.timeline()
    ctx.timeline_enable(False)
    names = ["attention", "qkv", "o", "gate_up", "down"]
    launches = sorted(set(rec["launch"].tolist()))
    mid = [L for L in launches if len(launches) // 4 <= launches.index(L) < 3 * len(launches) // 4]
    span = {}
    for L in mid:
        for k in range(5):
            r = rec[(rec["launch"] == L) & (rec["kind"] == k)]
            if len(r):
                span[(L, k)] = (float(r["t_ready"].min()) / rate, float(r["t_end"].max()) / rate, int(len(r)))
    dur = {names[k]: [e - b for (L, kk), (b, e, n) in span.items() if kk == k] for k in range(5)}
    att = sorted(L for (L, k) in span if k == 0)
    period = [span[(b, 0)][0] - span[(a, 0)][0] for a, b in zip(att, att[1:])]
    # phases of a ladder layer: launch L holds attention, gate/up and o; launch L + 1 the next layer's qkv and down
    ph_a = [max(span[(L, 2)][1], span[(L, 3)][1]) - min(span[(L, 0)][0], span[(L, 3)][0]) for L in att if (L, 2) in span and (L, 3) in span]
    ph_b = [max(span[(L + 1, 1)][1], span[(L + 1, 4)][1]) - min(span[(L + 1, 1)][0], span[(L + 1, 4)][0])
            for L in att if (L + 1, 1) in span and (L + 1, 4) in span]
    mean = lambda v: (sum(v) / len(v)) if v else None
    return {"unit": "us", "layers_averaged": len(att), "blocks_recorded": int(len(rec)),
            "period_per_layer": mean(period),
            "first_ready_to_last_end": {k: mean(v) for k, v in dur.items() if v},
            "phase_attention_o_beside_gate_up": mean(ph_a), "phase_qkv_beside_down": mean(ph_b),
            "note": "blocks taken from a launch's surplus list are not recorded"}


def run_decode_stages(args):
    """Decode steps through a pipeline of --stages contexts on the one GPU, each holding a run of the workload's layers
    and handing residual, attention output and MLP output to the next one in device memory (section "Compatibility
    with other Parallelism Techniques"): what the stage boundary costs beside the same layers in one context."""
    import torch
    from paper_2501_06589_amd import inputs, ladder
    w = inputs.WORKLOADS[args.workload]
    if args.layers:
        w = w.with_(n_layers=args.layers)
    if args.batch:
        w = w.with_(batch=args.batch)
    if args.kv and w.kv_preload:
        w = w.with_(kv_preload=args.kv)
    if not w.kv_preload:
        raise SystemExit("--stages needs a workload with a preloaded cache (70b_r8_decode)")
    dev = "cuda:0"
    total_steps = args.warmup + args.steps
    k = args.stages
    cuts = [(w.n_layers * s // k, w.n_layers * (s + 1) // k) for s in range(k)]
    plan = 0 if args.no_fused else {"paired": 1, "single": 2, "chain": 3}[args.fused_plan]
    stages = [build_context(w.with_(n_layers=b - a), dev, total_steps, w.batch, layer0=a, max_tokens=1, decode_fused=plan)
              for a, b in cuts]
    kv = [[inputs.kv_cache(w, i, r, w.batch, w.kv_preload, dev) for r in range(w.n_real_shards)] for i in range(w.n_layers)]

    def reset_cache():
        for s, (a, b) in enumerate(cuts):
            for i in range(a, b):
                for r in range(w.n_real_shards):
                    stages[s].load_kv(i - a, r, kv[i][r][0], kv[i][r][1])

    xs = torch.stack([inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0 + i, dev)[:, 0] for i in range(total_steps)]).float()
    out = None

    def step(i):
        nonlocal out
        hand = (xs[i], None, None)
        for ctx in stages:
            hand = ctx.decode_step_stage(hand)
        out = hand[0] + hand[1] + hand[2]          # x_2N

    rep_ms = []
    for rep in range(max(1, args.reps)):
        reset_cache()
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        rep_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)
        assert torch.isfinite(out).all()
    ms_per_step = sorted(rep_ms)[len(rep_ms) // 2]
    for ctx in stages:
        ctx.free()
    return {
        "metric": "decode_tokens_per_s", "value": w.batch / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "repetitions": {"n": len(rep_ms), "ms_per_step": rep_ms, "reported": "median"},
        "config": {"workload": w.name, "n_layers": w.n_layers, "batch": w.batch, "pipeline_stages": k, "layers_per_stage": [b - a for a, b in cuts],
                   "note": "all stages on the one GPU, one after the other; the hand-over stays in device memory"},
    }


def run_prefill(args):
    import torch
    from paper_2501_06589_amd import inputs, ladder
    w = inputs.WORKLOADS[args.workload]
    if args.layers:
        w = w.with_(n_layers=args.layers)
    if args.batch:
        w = w.with_(batch=args.batch)
    dev = "cuda:0"
    rows = w.batch * w.prefill
    ctx = build_context(w, dev, 8, rows)
    x = inputs.embeddings(w, w.batch, w.prefill, inputs.SEED_PREFILL, dev)
    out = torch.empty((w.batch, w.prefill, w.hidden), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] context ready: {ctx.device_bytes() / 2**30:.2f} GiB on device")
    for _ in range(args.warmup):
        ctx.prefill(x, out)
    torch.cuda.synchronize()
    call_ms = []
    for _ in range(args.steps):        # every call timed on its own; the median is reported
        t0 = time.perf_counter()
        ctx.prefill(x, out)
        torch.cuda.synchronize()
        call_ms.append((time.perf_counter() - t0) * 1e3)
    assert torch.isfinite(out).all()
    ms_per_step = sorted(call_ms)[len(call_ms) // 2]
    dt = ms_per_step * 1e-3 * args.steps
    gemm_flops = 2.0 * w.n_layers * w.n_real_shards * w.params_per_layer() * rows
    attn_flops = w.n_layers * w.n_real_shards * w.batch * w.n_q_heads * 4.0 * w.head_dim * (w.prefill * (w.prefill + 1) / 2)
    ctx.profile_enable(True)
    ctx.profile_reset()
    ctx.prefill(x, out)
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    n_gemm, ms_gemm = prof["gemm"]
    flops_per_launch = gemm_flops / (4 * w.n_layers * w.n_real_shards)
    avg_ms = ms_gemm / max(n_gemm, 1)
    achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12 if n_gemm else 0.0
    roofline = {"bound": "mfma", "kernel": "gemm_lds_kernel (prefill bf16 MFMA GEMM, 256 x 256 tiles)", "achieved": achieved,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": None, "algorithmic_flops_per_launch": flops_per_launch, "avg_launch_ms": avg_ms,
                "launches": n_gemm}
    per_class = {k: {"launches": n, "avg_us": (ms / n * 1e3 if n else 0.0), "ms_per_step": ms}
                 for k, (n, ms) in prof.items() if n}
    ctx.free()
    return {
        "metric": "prefill_tokens_per_s", "value": rows * args.steps / dt, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "repetitions": {"n": args.steps, "ms_per_call": call_ms, "reported": "median"},
        "config": {"workload": w.name, "n_layers": w.n_layers, "hidden": w.hidden, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "inter": w.inter, "tp_degree": w.tp_degree,
                   "batch": w.batch, "prefill_tokens": w.prefill, "peers": w.n_peers},
        "mfma": {"gemm_flops": gemm_flops, "attention_flops": attn_flops,
                 "whole_prefill_TFLOPs": (gemm_flops + attn_flops) / (ms_per_step * 1e-3) / 1e12,
                 "frac_of_peak_whole_prefill": (gemm_flops + attn_flops) / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "roofline": roofline, "kernel_classes": per_class, "cpu_baseline": None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--mode", choices=["both", "decode", "prefill"], default="both",
                    help="both (default): the decode workload, then the prefill workload, one JSON line carrying the two "
                         "halves of the metric; decode / prefill: that half alone (any workload)")
    ap.add_argument("--reps", type=int, default=3, help="decode: timed regions of --steps steps each (the median is reported)")
    ap.add_argument("--no-ceiling", action="store_true", help="decode: skip the copy-kernel measurement of the box's streaming rate")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--kv", type=int, default=0, help="override the preloaded cache length of a decode workload")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (1.2b / 8b are quoted at 1, 4, 16)")
    ap.add_argument("--layers", type=int, default=0, help="debug: truncate the stack (result is then not the metric)")
    ap.add_argument("--cpu-layers", type=int, default=32, help="layers of the oracle's timed sample")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--graph", action="store_true", help="replay decode steps from a captured HIP graph instead of eager launches")
    ap.add_argument("--no-overlap", action="store_true", help="one compute stream instead of attention / MLP streams")
    ap.add_argument("--wiring", choices=["ladder", "standard", "parallel"], default="ladder",
                    help="residual wiring of the stack (the metric is quoted on ladder; standard is the paper's Eq. 1 baseline)")
    ap.add_argument("--standard-layers", type=int, default=0,
                    help="hybrid stack: with --wiring ladder, the lower N layers keep the standard wiring (the paper's "
                         "Hybrid-Ladder-8B-16L is --workload 8b --standard-layers 16)")
    ap.add_argument("--no-peers", action="store_true",
                    help="no synthetic peer partial sums: with the standard wiring and no emulated latency this is the "
                         "communication-free upper bound of the paper's comparison (result is then not the metric)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="before the steps, run 4 plain copy kernels of 1 GiB (read 1 GiB, write 1 GiB each): "
                         "the known-size dispatches that scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--reduce-delay-us", type=int, default=0,
                    help="emulated all-reduce latency: every collective takes this long before the stream it completes may be read")
    ap.add_argument("--fused-plan", choices=["paired", "single", "chain"], default="chain",
                    help="fused decode schedule: chain = the paired launch list as ONE launch of persistent workgroups per "
                         "step, jobs meeting at completion flags (default); paired = independent jobs of neighbouring modules "
                         "share a launch; single = one job per launch (five per layer), which leaves each collective a module "
                         "to hide behind")
    ap.add_argument("--head", action="store_true",
                    help="decode mode: generate for real (token embedding -> stack -> final norm + output projection of "
                         "this rank's vocabulary slice -> greedy token, fed back); the metric is quoted without it")
    ap.add_argument("--no-fused", action="store_true", help="one kernel per operation instead of the fused decode launches")
    ap.add_argument("--timeline", action="store_true",
                    help="decode, chained step: add the library's timeline of one step (per kind of job and per phase of a layer)")
    ap.add_argument("--stages", type=int, default=0,
                    help="decode: the workload's layers as this many pipeline-stage contexts that hand residual, attention "
                         "output and MLP output to one another (ladder_decode_step_stage); prints the step time only")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (one process, one MI355X); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.mode in ("decode", "both"):
        both = args.mode == "both" and args.workload in (None, "70b_r8_decode")
        args.workload = args.workload or "70b_r8_decode"
        steps_given, warmup_given = args.steps, args.warmup
        args.steps = 256 if args.steps is None else args.steps
        args.warmup = 16 if args.warmup is None else args.warmup
        if args.stages > 0:
            print(json.dumps(run_decode_stages(args)))
            return
        res = run_decode(args)
        if both:
            # the other half of the metric: the prefill workload on a fresh context (the decode context has been freed)
            pa = argparse.Namespace(**vars(args))
            pa.workload, pa.steps, pa.warmup, pa.batch, pa.layers = "70b_r4_prefill", 3, 1, 0, args.layers
            pr = run_prefill(pa)
            res["prefill"] = {"workload": pr["config"]["workload"], "rows": pr["config"]["batch"] * pr["config"]["prefill_tokens"],
                              "ms": pr["ms_per_step"], "ms_per_call": pr["repetitions"]["ms_per_call"], "tokens_per_s": pr["value"],
                              "gemm_tflops": pr["roofline"]["achieved"], "gemm_frac": pr["roofline"]["frac"],
                              "whole_tflops": pr["mfma"]["whole_prefill_TFLOPs"], "whole_frac": pr["mfma"]["frac_of_peak_whole_prefill"],
                              "peak_tflops": MFMA_BF16_PEAK_TFLOPS, "dtype": "bf16", "kernel_classes": pr["kernel_classes"],
                              "roofline": pr["roofline"]}
    else:
        args.workload = args.workload or "70b_r4_prefill"
        args.steps = 3 if args.steps is None else args.steps
        args.warmup = 1 if args.warmup is None else args.warmup
        res = run_prefill(args)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
