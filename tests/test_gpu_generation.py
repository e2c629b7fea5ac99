"""GPU parity of the generation head (token embedding, final RMSNorm + output projection, greedy
sampling) and of a prefill-then-decode generation loop through the C-ABI, against oracle/generation.py."""
import numpy as np
import pytest
import torch

from oracle import from_torch, generation as gen
from oracle import ladder_oracle as lo
from paper_2501_06589_amd import inputs, ladder

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TINY = inputs.WORKLOADS["tiny"]
SMALL_BF16 = TINY.with_(name="small_bf16_gen", dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, inter=352,
                        tp_degree=1, n_real_shards=1, batch=3, prefill=24, decode_steps=5)


@pytest.fixture(scope="module")
def harness():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def _setup(harness, w, vocab, vocab_local=None):
    tensors = harness.make_tensors(w)
    ctx = harness.build_gpu(w, tensors, None)
    head = inputs.head_weights(w, vocab, vocab_local)
    ctx.load_head(*(head[k].to(DEV) for k in ("table", "final_norm", "w_lm")))
    cfg = from_torch.config_from_workload(w)
    layers = [from_torch.layer_from_tensors(tensors[i]) for i in range(w.n_layers)]
    ohead = {k: from_torch.to_f64(v) for k, v in head.items()}
    return ctx, cfg, layers, ohead


def _check_tokens(got_tokens, ref_logits, slack):
    """The sampled index is the oracle's arg max, or, where the oracle's best two are closer than the
    comparison tolerance, one whose oracle logit is within that slack of the maximum."""
    for r, t in enumerate(got_tokens):
        assert 0 <= t < ref_logits.shape[1]
        assert ref_logits[r, t] >= ref_logits[r].max() - slack, (r, t, int(np.argmax(ref_logits[r])))


@pytest.mark.parametrize("w,vocab,vocab_local,tol", [(TINY.with_(name="tiny_gen", batch=2, prefill=8, decode_steps=6), 200, None, 1e-4),
                                                     (SMALL_BF16, 512, 256, 2e-2)])
def test_generation_loop_matches_oracle(harness, w, vocab, vocab_local, tol):
    """Prefill a seeded prompt, then decode; at every step both sides are fed the oracle's token (so one
    near-tie cannot send the two sequences apart) and the logits of the step are compared element by
    element; the GPU's own greedy choice is checked against the oracle's logits."""
    ctx, cfg, layers, oh = _setup(harness, w, vocab, vocab_local)
    prompt = inputs.prompt_tokens(w.batch, w.prefill, vocab)
    state = lo.State.empty(cfg, w.n_real_shards, w.batch, w.prefill + w.decode_steps)
    # embedding: a row gather, bit exact
    emb = ctx.embed(prompt.to(DEV))
    want_emb = gen.embed(prompt.numpy(), oh["table"])
    assert np.array_equal(emb.float().cpu().double().numpy(), want_emb)
    x = ctx.prefill(emb)
    ref_x = lo.forward_eq2(want_emb, layers, cfg, state)
    errs = []
    for step in range(w.decode_steps):
        logits, toks = ctx.head(x[:, -1].contiguous() if x.dim() == 3 else x)
        ref_logits = gen.lm_head(ref_x[:, -1], oh["final_norm"], oh["w_lm"], cfg.rms_eps)
        rms = np.sqrt(np.mean(ref_logits ** 2))
        got = logits.cpu().double().numpy()
        errs.append(float(np.max(np.abs(got - ref_logits)) / rms))
        _check_tokens(toks.cpu().numpy(), ref_logits, 2 * tol * rms)
        assert np.array_equal(toks.cpu().numpy(), np.argmax(got, axis=-1))      # the kernel's arg max of its own logits
        nxt = gen.greedy(ref_logits) % vocab                                     # teacher forcing with the oracle's token
        nxt_t = torch.from_numpy(nxt.astype(np.int32))
        x = ctx.decode_step(ctx.embed(nxt_t.to(DEV)))[:, None, :]
        ref_x = lo.forward_eq2(gen.embed(nxt[:, None], oh["table"]), layers, cfg, state)
    print(f"[gen] {w.name}: logits max err / rms per step = {['%.2e' % e for e in errs]}", flush=True)
    assert max(errs) < tol, errs
    ctx.free()


def test_greedy_tie_takes_the_lowest_index_and_errors(harness):
    w = TINY.with_(name="tiny_gen_tie", batch=2, prefill=4)
    tensors = harness.make_tensors(w)
    ctx = harness.build_gpu(w, tensors, None)
    x = torch.randn((2, w.hidden), device=DEV)
    with pytest.raises(ladder.LadderError) as e:
        ctx._vocab_local = 8
        ctx.head(x)                                          # head not loaded
    assert e.value.code == ladder.LADDER_E_STATE
    head = inputs.head_weights(w, 64)
    wl = head["w_lm"].clone()
    wl[:, 40] = wl[:, 7]                                      # two identical columns: identical logits
    wl[:, 7] *= 0
    wl[:, 40] *= 0
    wl[:, 7] += 10.0 * head["w_lm"][:, 3].abs().max()         # make them the maximum for any positive-sum row
    wl[:, 40] = wl[:, 7]
    ctx.load_head(head["table"].to(DEV), torch.ones_like(head["final_norm"]).to(DEV), wl.to(DEV))
    xp = torch.rand((2, w.hidden), device=DEV) + 0.5           # positive rows -> columns 7 and 40 tie at the top
    logits, toks = ctx.head(xp)
    lg = logits.cpu().numpy()
    assert np.array_equal(lg[:, 7], lg[:, 40]) and np.all(lg[:, 7] >= lg.max(axis=1))
    assert toks.cpu().tolist() == [7, 7]
    with pytest.raises(ladder.LadderError) as e:
        ctx.head(torch.zeros((3, w.hidden), device=DEV))     # more rows than max_batch
    assert e.value.code == ladder.LADDER_E_SHAPE
    with pytest.raises(ladder.LadderError) as e:
        ctx.load_head(head["table"].to(DEV), head["final_norm"].to(DEV), head["w_lm"].to(DEV))   # twice
    assert e.value.code == ladder.LADDER_E_STATE
    ctx.free()


def test_token_id_outside_the_table_is_reported_by_the_next_call(harness):
    """ladder_embed never reads outside its table, and says so afterwards: the call that meets the bad id returns
    LADDER_OK (it had only been enqueued); once its kernel has run, the next call reports LADDER_E_ARG once."""
    w = TINY.with_(name="tiny_gen_oor", batch=2, prefill=4)
    ctx, cfg, layers, oh = _setup(harness, w, 50)
    good = torch.tensor([[1, 2, 3, 4], [5, 6, 7, 49]], dtype=torch.int32, device=DEV)
    ctx.embed(good)
    torch.cuda.synchronize()
    ctx.embed(good)                                             # nothing to report
    bad = torch.tensor([[1, 2, 50, 4], [5, -1, 7, 8]], dtype=torch.int32, device=DEV)
    emb = ctx.embed(bad)                                        # rows of the nearest valid ids, no fault
    torch.cuda.synchronize()
    want = gen.embed(np.clip(bad.cpu().numpy(), 0, 49), oh["table"])
    assert np.array_equal(emb.float().cpu().double().numpy(), want)
    with pytest.raises(ladder.LadderError) as e:
        ctx.prefill(emb)
    assert e.value.code == ladder.LADDER_E_ARG and "token id" in str(e.value)
    assert ctx.position() == (0, 0)
    ctx.prefill(ctx.embed(good))                                # reported once; normal operation again
    torch.cuda.synchronize()
    assert ctx.position() == (4, 2)
    ctx.free()
