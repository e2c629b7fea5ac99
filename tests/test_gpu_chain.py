"""GPU parity of the chained decode step (decode_fused = 3): the whole launch list of a step in one launch of
persistent workgroups, the jobs meeting at flags instead of launch boundaries.  The arithmetic and its order are
those of the launch list, so the results are bit-identical to the launch-per-job schedules; against the oracle the
bar is the bf16-storage one (max |gpu - oracle| / RMS(oracle) < 2e-2 on every call's final x_2N).
"""
import numpy as np
import pytest
import torch

from paper_2501_06589_amd import inputs, ladder

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
R8_SMALL = inputs.WORKLOADS["70b_r8_decode"].with_(name="r8_small", n_layers=3, hidden=512, inter=448, batch=4,
                                                   decode_steps=6)


@pytest.fixture(scope="module")
def harness():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("wiring,nstd", [(ladder.LADDER_WIRING_LADDER, 0), (ladder.LADDER_WIRING_STANDARD, 0),
                                         (ladder.LADDER_WIRING_LADDER, 2), (ladder.LADDER_WIRING_PARALLEL, 0)])
def test_chained_step_matches_oracle_and_the_launch_list(harness, wiring, nstd):
    """Every wiring (Algorithm 1, Eq. 1, the hybrid stack, the parallel block), synthetic peers, preloaded cache,
    decode crossing a 32-position boundary: against the oracle, and bit for bit against the same launch list run
    as separate launches."""
    kw = dict(kv_preload=125 if nstd else 700, wiring=wiring, n_standard_layers=nstd)
    res = harness.run_case(R8_SMALL, decode_fused=3, **kw)
    assert len(res.errs) == 6 and max(res.errs) < TOL_BF16, res.errs
    ref = harness.run_case(R8_SMALL, gpu_only=True, decode_fused=1, **kw)
    for x, y in zip(res.gpu, ref.gpu):
        assert np.array_equal(x, y)


def test_chained_step_graph_replay_eager_and_rerun_bit_identical(harness):
    a = harness.run_case(R8_SMALL, kv_preload=125, gpu_only=True, decode_fused=3, decode_graph=0)
    b = harness.run_case(R8_SMALL, kv_preload=125, gpu_only=True, decode_fused=3, decode_graph=1)
    c = harness.run_case(R8_SMALL, kv_preload=125, gpu_only=True, decode_fused=3, decode_graph=0)
    for x, y, z in zip(a.gpu, b.gpu, c.gpu):
        assert np.array_equal(x, y) and np.array_equal(x, z)


def test_chained_step_other_geometries(harness):
    """d = 64 with 2 q heads per kv head, batch 2, after a real prefill; batch 16 (two MFMA operands per k tile)
    with d = 128, 4 per group; batch 14 with four-tile gate/up workgroups; a single sequence."""
    small = inputs.WORKLOADS["tiny"].with_(name="small_bf16_chain", dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2,
                                           head_dim=64, inter=352, tp_degree=1, n_real_shards=1, batch=2, prefill=40,
                                           decode_steps=4)
    res = harness.run_case(small, decode_fused=3)
    assert max(res.errs) < TOL_BF16, res.errs
    w = inputs.WORKLOADS["70b_r4_prefill"].with_(name="r4_b16_chain", n_layers=2, hidden=512, n_q_heads=8, n_kv_heads=2,
                                                 inter=512, batch=16, prefill=0, kv_preload=70, decode_steps=3)
    res = harness.run_case(w, kv_preload=70, decode_fused=3)
    assert max(res.errs) < TOL_BF16, res.errs
    w = R8_SMALL.with_(name="r8_small_gu4_chain", inter=8704, batch=14, decode_steps=3)
    res = harness.run_case(w, kv_preload=100, decode_fused=3)
    assert len(res.errs) == 3 and max(res.errs) < TOL_BF16, res.errs
    w = R8_SMALL.with_(name="r8_small_b1_chain", batch=1, decode_steps=3)
    res = harness.run_case(w, kv_preload=100, decode_fused=3)
    assert len(res.errs) == 3 and max(res.errs) < TOL_BF16, res.errs


@pytest.mark.parametrize("kv,batch,nq,nkv,d", [(2300, 2, 8, 1, 128), (5000, 3, 4, 2, 64), (9000, 1, 8, 1, 128)])
def test_chained_step_long_context_split_attention(harness, kv, batch, nq, nkv, d):
    """Caches of thousands of positions: many attention splits per (sequence, kv head), merged by the last to
    arrive, inside the one launch; three steps, so that tickets and completion words are used again."""
    w = inputs.WORKLOADS["70b_r8_decode"].with_(name=f"long_ctx_chain_{kv}", n_layers=2, hidden=256, inter=256, n_q_heads=nq,
                                                n_kv_heads=nkv, head_dim=d, batch=batch, prefill=0, kv_preload=kv,
                                                decode_steps=3)
    res = harness.run_case(w, kv_preload=kv, decode_fused=3)
    assert len(res.errs) == 3 and max(res.errs) < TOL_BF16, res.errs
    ref = harness.run_case(w, kv_preload=kv, gpu_only=True, decode_fused=1)
    for x, y in zip(res.gpu, ref.gpu):
        assert np.array_equal(x, y)


def test_chained_step_launches_with_more_blocks_than_slots(harness):
    """A launch list whose launches have more blocks than the device has workgroup slots (512 pairs of gate/up tiles +
    128 workgroups of the output projection + attention against 512 slots): the blocks beyond the slots sit in the
    launch's surplus list and are taken by whichever slot gets there first.  Which slot runs a block changes nothing in
    its arithmetic, nor does it that the chained step takes the gate/up tiles in pairs where separate launches take
    them one by one: against the oracle, bit for bit against separate launches, and the same bits again on a second run."""
    w = R8_SMALL.with_(name="r8_surplus_chain", n_layers=2, hidden=4096, inter=8192, batch=8, decode_steps=3)
    res = harness.run_case(w, kv_preload=300, decode_fused=3)
    assert len(res.errs) == 3 and max(res.errs) < TOL_BF16, res.errs
    ref = harness.run_case(w, kv_preload=300, gpu_only=True, decode_fused=1)
    again = harness.run_case(w, kv_preload=300, gpu_only=True, decode_fused=3, decode_graph=1)
    for x, y, z in zip(res.gpu, ref.gpu, again.gpu):
        assert np.array_equal(x, y) and np.array_equal(x, z)
    # the timeline records the blocks that were dealt out beforehand only: fewer gate/up tiles than the layers have
    tensors = harness.make_tensors(w)
    ctx = harness.build_gpu(w, tensors, inputs.peer_partials(w, w.batch), max_seq=400, decode_fused=3)
    for i in range(w.n_layers):
        k, v = inputs.kv_cache(w, i, 0, w.batch, 50)
        ctx.load_kv(i, 0, k.to("cuda:0"), v.to("cuda:0"))
    x = inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0)[:, 0].contiguous().to("cuda:0")
    ctx.timeline_enable(True)
    ctx.decode_step(x)
    rec, _ = ctx.timeline()
    gu = rec[rec["kind"] == 3]
    assert 0 < gu["tiles"].sum() < 2 * w.inter // 16 * w.n_layers, gu["tiles"].sum()
    assert rec["slot"].max() + 1 == 2 * torch.cuda.get_device_properties(0).multi_processor_count
    ctx.free()


def test_chained_step_with_emulated_collective_latency_same_bits(harness):
    """reduce_delay_us on a chained step: the projections that read a stream hold back until its emulated
    collective is over; the arithmetic does not change."""
    kw = dict(kv_preload=125, gpu_only=True, decode_fused=3)
    base = harness.run_case(R8_SMALL, **kw)
    late = harness.run_case(R8_SMALL, reduce_delay_us=100, **kw)
    for x, y in zip(base.gpu, late.gpu):
        assert np.array_equal(x, y)


def test_timeline_of_a_chained_step(harness):
    """The timeline's records: one per block of the launch list, times in order, and no block ready before the
    blocks of the launch that produces its input have ended (ladder wiring: down_l after gate/up_l, o_l after
    attention_l, QKV_{l+1} after o_l)."""
    w = R8_SMALL
    tensors = harness.make_tensors(w)
    ctx = harness.build_gpu(w, tensors, inputs.peer_partials(w, w.batch), max_seq=200, decode_fused=3)
    for i in range(w.n_layers):
        k, v = inputs.kv_cache(w, i, 0, w.batch, 50)
        ctx.load_kv(i, 0, k.to("cuda:0"), v.to("cuda:0"))
    x = inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0)[:, 0].contiguous().to("cuda:0")
    with pytest.raises(ladder.LadderError):
        ctx.timeline()                       # nothing enabled yet
    ref = ctx.decode_step(x).cpu()
    ctx.timeline_enable(True)
    ctx.decode_step(x)
    rec, rate = ctx.timeline()
    assert rate > 0 and len(rec) > 0
    assert np.all(rec["t_take"] <= rec["t_ready"]) and np.all(rec["t_ready"] <= rec["t_end"]) and np.all(rec["t_take"] > 0)
    kinds = {k: rec[rec["kind"] == k] for k in range(5)}
    n_tiles = {1: (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim // 16, 2: w.hidden // 16, 3: 2 * w.inter // 16, 4: w.hidden // 16}
    for k, per_layer in n_tiles.items():
        assert kinds[k]["tiles"].sum() == per_layer * w.n_layers, (k, kinds[k]["tiles"].sum())
    by_launch = lambda k, L: kinds[k][kinds[k]["launch"] == L]
    launches = sorted(set(rec["launch"]))
    for L in launches:
        att, o = by_launch(0, L), by_launch(2, L)
        if len(att) and len(o):              # { attention_l, gate/up_l, o_l }
            assert o["t_ready"].min() >= att["t_end"].min()
            gu, dn, qkv = by_launch(3, L), by_launch(4, L + 1), by_launch(1, L + 1)
            if len(dn):
                assert dn["t_ready"].min() >= gu["t_end"].max() and dn["t_ready"].min() >= o["t_end"].max()
            if len(qkv):
                assert qkv["t_ready"].min() >= o["t_end"].max()
    ctx.timeline_enable(False)
    out = ctx.decode_step(x).cpu()
    assert torch.isfinite(out).all() and ref.shape == out.shape
    ctx.free()
