"""Runs one seeded case through the HIP library (C-ABI via the ctypes binding) and through the CPU
oracle on the same inputs; used by the GPU parity tests."""
from __future__ import annotations

import sys
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from oracle import from_torch
from oracle import ladder_oracle as lo
from paper_2501_06589_amd import inputs, ladder

DEV = "cuda:0"


@dataclass
class CaseResult:
    errs: List[float]           # max|gpu - oracle| / rms(oracle) per call (prefill first, then decode steps)
    gpu: List[np.ndarray]
    ref: List[np.ndarray]


def say(msg: str):
    print(msg, flush=True)
    sys.stdout.flush()


def build_gpu(w: inputs.Workload, tensors, peers=None, **cfg_override) -> ladder.Ladder:
    ctx = ladder.Ladder(ladder.config_for(w, **cfg_override))
    for i in range(w.n_layers):
        for r in range(w.n_real_shards):
            ctx.load_layer(i, r, {k: v.to(DEV) for k, v in tensors[i][r].items()})
    if peers is not None:
        ctx.set_peer_partials(peers.to(DEV))
    torch.cuda.synchronize()
    return ctx


def make_tensors(w: inputs.Workload, device="cpu"):
    return [[inputs.layer_weights(w, i, r, device) for r in range(w.n_real_shards)] for i in range(w.n_layers)]


def oracle_lag(w: inputs.Workload, wiring: int, n_standard_layers: int):
    if wiring == ladder.LADDER_WIRING_STANDARD:
        return "standard"
    if wiring == ladder.LADDER_WIRING_PARALLEL:
        return "parallel"
    if n_standard_layers == 0:
        return "ladder"
    return [1 if (m - 1) // 2 < n_standard_layers else 2 for m in range(1, 2 * w.n_layers + 1)]


def run_case(w: inputs.Workload, *, decode_steps: Optional[int] = None, kv_preload: int = 0,
             wiring: int = ladder.LADDER_WIRING_LADDER, n_standard_layers: int = 0, use_peers: bool = True,
             gpu_only: bool = False, tensors=None, gen_device: str = "cpu", **cfg_override) -> CaseResult:
    """Prefill (or synthetic cache preload) then decode steps on both sides.  Every input is generated
    once, on gen_device, and copied to the side that does not have it (full-width cases generate on the
    GPU, where the seeded generator takes seconds, and build the oracle's float64 layers one at a time)."""
    steps = w.decode_steps if decode_steps is None else decode_steps
    say(f"[case] {w.name} dtype={w.dtype} L={w.n_layers} H={w.hidden} nq/nkv={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim} "
        f"I={w.inter} R={w.tp_degree}/{w.n_real_shards} B={w.batch} T={w.prefill} kv={kv_preload} steps={steps} "
        f"wiring={wiring}/{n_standard_layers} cfg={cfg_override}")
    tensors = tensors or make_tensors(w, gen_device)
    rows = w.batch * max(w.prefill, 1)
    peers = inputs.peer_partials(w, rows, gen_device) if (use_peers and w.n_peers) else None
    ctx = build_gpu(w, tensors, peers, wiring=wiring, n_standard_layers=n_standard_layers, **cfg_override)
    cfg = from_torch.config_from_workload(w)
    def oracle_layer(i):
        return from_torch.layer_from_tensors([{k: v.cpu() for k, v in t.items()} for t in tensors[i]])
    layers = (from_torch.LazyLayers(w.n_layers, oracle_layer) if gen_device != "cpu"
              else [oracle_layer(i) for i in range(w.n_layers)])
    state = lo.State.empty(cfg, w.n_real_shards, w.batch, w.max_seq + kv_preload)
    opeers = from_torch.to_f64(peers.cpu()) if peers is not None else None
    lag = oracle_lag(w, wiring, n_standard_layers)
    gpu_out, ref_out = [], []
    if kv_preload:
        for i in range(w.n_layers):
            for r in range(w.n_real_shards):
                k, v = inputs.kv_cache(w, i, r, w.batch, kv_preload, gen_device)
                ctx.load_kv(i, r, k.to(DEV), v.to(DEV))
                from_torch.load_kv(state, i, r, k.cpu(), v.cpu())
        state.pos = kv_preload
    else:
        emb = inputs.embeddings(w, w.batch, w.prefill, inputs.SEED_PREFILL, gen_device)
        gpu_out.append(ctx.prefill(emb.to(DEV)).cpu().double().numpy())
        if not gpu_only:
            ref_out.append(lo.forward_eq2(from_torch.to_f64(emb.cpu()), layers, cfg, state, opeers, wiring=lag))
    for step in range(steps):
        e = inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0 + step, gen_device)
        gpu_out.append(ctx.decode_step(e[:, 0].contiguous().to(DEV)).cpu().double().numpy()[:, None, :])
        if not gpu_only:
            ref_out.append(lo.forward_eq2(from_torch.to_f64(e.cpu()), layers, cfg, state, opeers, wiring=lag))
    torch.cuda.synchronize()
    pos, batch = ctx.position()
    assert batch == w.batch and pos == (kv_preload or w.prefill) + steps
    ctx.free()
    errs = []
    for g, r in zip(gpu_out, ref_out):
        assert g.shape == r.shape, (g.shape, r.shape)
        assert np.all(np.isfinite(g)), ("non-finite", int(np.sum(~np.isfinite(g))), g.size)
        errs.append(float(np.max(np.abs(g - r)) / np.sqrt(np.mean(r * r))))
    rms_errs = [float(np.sqrt(np.mean((g - r) ** 2) / np.mean(r * r))) for g, r in zip(gpu_out, ref_out)]
    say(f"[case] {w.name}: max errs = {['%.2e' % v for v in errs]} rms errs = {['%.2e' % v for v in rms_errs]}")
    return CaseResult(errs, gpu_out, ref_out)
