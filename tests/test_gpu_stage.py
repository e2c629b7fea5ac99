"""GPU parity of the pipeline-stage entry points (section "Compatibility with other Parallelism Techniques"): a
context that holds some of a model's layers takes the three tensors Algorithm 1 passes from block to block
(residual, attention output, MLP output) and leaves the same three for the next stage.

Checked per call and per stage against the oracle's `stage_alg1` (fed with the oracle's own hand-over, so that a
stage's error is its own), tensor by tensor: max |gpu - oracle| over the RMS of the stage's stream (the sum of the
three) stays under the storage type's bar; the sum of the last stage's tensors is held against the oracle's x_2N and
against the same model run as ONE context through ladder_prefill / ladder_decode_step.
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2501_06589_amd import inputs, ladder

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_FP32 = 1e-4
DEV = "cuda:0"


@pytest.fixture(scope="module")
def harness():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def run_stages(harness, w, cuts, *, kv_preload=0, steps=3, gen_device="cpu", **cfg_override):
    """The model of workload `w` as one context and as the stages `cuts` = [(first layer, end layer), ...]; returns
    per call: (per stage [(gpu three, oracle three)], gpu x_2N of the one context, oracle x_2N)."""
    from oracle import from_torch
    from oracle import ladder_oracle as lo
    harness.say(f"[stage case] {w.name} L={w.n_layers} cuts={cuts} kv={kv_preload} T={w.prefill} steps={steps} cfg={cfg_override}")
    tensors = harness.make_tensors(w, gen_device)     # (full-width cases generate on the GPU: seconds instead of minutes)
    rows = w.batch * max(w.prefill, 1)
    peers = inputs.peer_partials(w, rows, gen_device) if w.n_peers else None
    whole = harness.build_gpu(w, tensors, peers, **cfg_override)
    stages = [harness.build_gpu(w.with_(n_layers=j - i), tensors[i:j], peers, **cfg_override) for i, j in cuts]
    cfg = from_torch.config_from_workload(w)
    layers = [from_torch.layer_from_tensors([{k: v.cpu() for k, v in t.items()} for t in tensors[i]]) for i in range(w.n_layers)]
    opeers = from_torch.to_f64(peers.cpu()) if peers is not None else None
    o_whole = lo.State.empty(cfg, w.n_real_shards, w.batch, w.max_seq + kv_preload)
    o_cfgs = [dataclasses.replace(cfg, n_layers=j - i) for i, j in cuts]
    o_states = [lo.State.empty(c, w.n_real_shards, w.batch, w.max_seq + kv_preload) for c in o_cfgs]
    if kv_preload:
        for i in range(w.n_layers):
            s = next(k for k, (a, b) in enumerate(cuts) if a <= i < b)
            for r in range(w.n_real_shards):
                k, v = inputs.kv_cache(w, i, r, w.batch, kv_preload, gen_device)
                whole.load_kv(i, r, k.to(DEV), v.to(DEV))
                stages[s].load_kv(i - cuts[s][0], r, k.to(DEV), v.to(DEV))
                from_torch.load_kv(o_whole, i, r, k.cpu(), v.cpu())
                from_torch.load_kv(o_states[s], i - cuts[s][0], r, k.cpu(), v.cpu())
        o_whole.pos = kv_preload
        for st in o_states:
            st.pos = kv_preload
    calls = []
    if not kv_preload:
        calls.append(("prefill", inputs.embeddings(w, w.batch, w.prefill, inputs.SEED_PREFILL, gen_device)))
    for step in range(steps):
        calls.append(("decode", inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0 + step, gen_device)))
    out = []
    for kind, emb in calls:
        harness.say(f"[stage case] {kind} {tuple(emb.shape)}")
        e64 = from_torch.to_f64(emb.cpu())
        if kind == "prefill":
            x_whole = whole.prefill(emb.to(DEV)).cpu().double().numpy()
            hand = (emb.float().to(DEV), None, None)
        else:
            x_whole = whole.decode_step(emb[:, 0].contiguous().to(DEV)).cpu().double().numpy()[:, None, :]
            hand = (emb[:, 0].float().contiguous().to(DEV), None, None)
        o_hand = (e64, None, None)
        per_stage = []
        for s, ctx in enumerate(stages):
            hand = ctx.prefill_stage(hand) if kind == "prefill" else ctx.decode_step_stage(hand)
            o_hand = lo.stage_alg1(*o_hand, layers[cuts[s][0]:cuts[s][1]], o_cfgs[s], o_states[s], opeers,
                                   module_offset=2 * cuts[s][0])
            got = [t.cpu().double().numpy().reshape(o_hand[0].shape) for t in hand]
            per_stage.append((got, o_hand))
            # the next stage is fed what the GPU stage left; the oracle what the oracle stage left
        x_ref = lo.forward_eq2(e64, layers, cfg, o_whole, opeers)
        out.append((per_stage, x_whole, x_ref))
    torch.cuda.synchronize()
    for ctx in stages + [whole]:
        pos, batch = ctx.position()
        assert batch == w.batch and pos == (kv_preload or w.prefill) + steps
        ctx.free()
    return out


def check(harness, out, tol, what):
    for n, (per_stage, x_whole, x_ref) in enumerate(out):
        scale = float(np.sqrt(np.mean(x_ref * x_ref)))
        for s, (got, want) in enumerate(per_stage):
            sc = float(np.sqrt(np.mean(sum(want) ** 2)))
            errs = [float(np.max(np.abs(g - r)) / sc) for g, r in zip(got, want)]
            own = [float(np.sqrt(np.mean(r * r)) / sc) for r in want]
            harness.say(f"[stage] {what} call {n} stage {s}: max err / stream rms (residual, attn, mlp) = "
                        f"{['%.2e' % e for e in errs]}; the tensors' own rms / stream rms = {['%.2f' % o for o in own]}")
            assert all(np.all(np.isfinite(g)) for g in got)
            assert max(errs) < tol, (what, n, s, errs)
            # (the two outputs are far enough apart for a swap to fail the bar)
            assert float(np.max(np.abs(want[1] - want[2])) / sc) > 10 * tol
        total = sum(per_stage[-1][0])
        e_ref = float(np.max(np.abs(total - x_ref)) / scale)
        e_one = float(np.max(np.abs(total - x_whole)) / scale)
        e_whole = float(np.max(np.abs(x_whole - x_ref)) / scale)
        harness.say(f"[stage] {what} call {n}: sum of the last hand-over vs oracle x_2N {e_ref:.2e}, vs one context {e_one:.2e} "
                    f"(one context vs oracle {e_whole:.2e})")
        assert e_ref < tol and e_one < tol, (what, n, e_ref, e_one)


R8_STAGED = inputs.WORKLOADS["70b_r8_decode"].with_(name="r8_staged", n_layers=5, hidden=512, inter=448, batch=4, decode_steps=3)


@pytest.mark.parametrize("fused", [3, 1, 0])
def test_decode_stages_match_oracle_and_one_context(harness, fused):
    """Five layers cut 2 + 1 + 2 (a one-layer stage: its hand-over reaches back to its own input), synthetic peers,
    preloaded caches, decode steps in the chained step, the launch list and the per-operation schedule."""
    out = run_stages(harness, R8_STAGED, [(0, 2), (2, 3), (3, 5)], kv_preload=200, steps=3, decode_fused=fused)
    check(harness, out, TOL_BF16, f"decode_fused={fused}")


def test_decode_stages_full_width_70b_r8(harness):
    """The headline shard's real width (hidden 8192, 8 q / 1 kv heads, intermediate 3584, batch 4, 7 peers, 1024
    cached positions), two layers as two stages of one layer each, chained step."""
    w = inputs.WORKLOADS["70b_r8_decode"].with_(name="r8_full_width_staged", n_layers=2, decode_steps=2)
    out = run_stages(harness, w, [(0, 1), (1, 2)], kv_preload=w.kv_preload, steps=2, gen_device=DEV, decode_fused=3)
    check(harness, out, TOL_BF16, "70B R = 8 width")


def test_prefill_then_decode_stages_bf16(harness):
    """A prefill wide enough for the GEMM path with the residual epilogue (more than 64 rows), then decode steps."""
    w = R8_STAGED.with_(name="r8_staged_prefill", n_layers=4, batch=2, prefill=160, kv_preload=0, decode_steps=2)
    out = run_stages(harness, w, [(0, 2), (2, 4)], steps=2)
    check(harness, out, TOL_BF16, "bf16 prefill + decode")


def test_stages_fp32_two_real_shards(harness):
    """The fp32 storage path with both shards computed: the hand-over itself (sums and differences of fp32 streams)
    to the fp32 bar."""
    w = inputs.WORKLOADS["tiny"].with_(name="tiny_staged", n_layers=4, decode_steps=2)
    out = run_stages(harness, w, [(0, 1), (1, 4)], steps=2)
    check(harness, out, TOL_FP32, "fp32")


def test_stage_calls_reject_what_they_cannot_do(harness):
    w = R8_STAGED.with_(name="r8_stage_errors", n_layers=2)
    tensors = harness.make_tensors(w)
    for kw in (dict(wiring=ladder.LADDER_WIRING_STANDARD), dict(n_standard_layers=1), dict(wiring=ladder.LADDER_WIRING_PARALLEL)):
        ctx = harness.build_gpu(w, tensors, None, **kw)
        x = torch.zeros((w.batch, 1, w.hidden), dtype=torch.float32, device=DEV)
        with pytest.raises(ladder.LadderError) as e:
            ctx.prefill_stage((x, None, None))
        assert e.value.code == ladder.LADDER_E_STATE
        ctx.free()
    ctx = harness.build_gpu(w, tensors, None)
    x = torch.zeros((w.batch, w.hidden), dtype=torch.float32, device=DEV)
    with pytest.raises(ladder.LadderError) as e:
        ctx.decode_step_stage((x[:1], None, None))      # no cache yet (the binding sizes its check for one row then)
    assert e.value.code == ladder.LADDER_E_STATE
    lib = ladder.lib()
    p = x.data_ptr()
    assert lib.ladder_decode_step_stage(ctx._h, None, None, None, p, p, p) == ladder.LADDER_E_ARG
    assert lib.ladder_decode_step_stage(ctx._h, p, None, None, p, p, p) == ladder.LADDER_E_ARG       # outputs coincide
    assert lib.ladder_prefill_stage(ctx._h, p + 4, None, None, 1, 1, p, p + 4096, p + 8192) == ladder.LADDER_E_ARG   # alignment
    ctx.free()
