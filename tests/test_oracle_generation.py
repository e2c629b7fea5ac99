"""Pins of the generation oracle (oracle/generation.py): token embedding, final norm + output
projection, greedy sampling, and the prefill-then-decode loop.  CPU only.  Each pin checks against
something other than the oracle's own code: torch float64 library routines, numpy's argmax, a full
recompute without a cache; the planted mistakes at the end must each break a pin."""
import numpy as np
import pytest
import torch

from oracle import from_torch, generation as gen
from oracle import ladder_oracle as lo
from paper_2501_06589_amd import inputs

import helpers

TINY = inputs.WORKLOADS["tiny"]
VOCAB = 96


def _head(w=TINY, vocab=VOCAB):
    h = inputs.head_weights(w, vocab)
    return {k: from_torch.to_f64(v) for k, v in h.items()}


def test_embed_is_a_row_gather_like_torch_embedding():
    rng = np.random.default_rng(0)
    table = rng.standard_normal((17, 5))
    tok = rng.integers(0, 17, size=(3, 4))
    want = torch.nn.functional.embedding(torch.from_numpy(tok), torch.from_numpy(table)).numpy()
    assert np.array_equal(gen.embed(tok, table), want)
    with pytest.raises(ValueError):
        gen.embed(np.array([[17]]), table)
    with pytest.raises(ValueError):
        gen.embed(np.array([[-1]]), table)


def test_lm_head_is_rms_norm_then_matmul_and_splits_over_the_vocabulary():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 32)) * 3.0
    gain = 1.0 + 0.1 * rng.standard_normal(32)
    w = rng.standard_normal((32, 40)) * 0.05
    got = gen.lm_head(x, gain, w, 1e-5)
    tx = torch.from_numpy(x)
    want = (torch.nn.functional.rms_norm(tx, (32,), torch.from_numpy(gain), 1e-5) @ torch.from_numpy(w)).numpy()
    assert helpers.rel_err(got, want) < 1e-12
    # vocabulary-parallel: the ranks' slices of W_lm give the slices of the logits, nothing to reduce
    parts = [gen.lm_head(x, gain, w[:, r * 10:(r + 1) * 10], 1e-5) for r in range(4)]
    assert helpers.rel_err(np.concatenate(parts, axis=-1), got) < 1e-13
    # a constant row: rmsnorm gives gain * sign, so the logits are gain . W (closed form)
    const = np.full((1, 32), 2.5)
    assert helpers.rel_err(gen.lm_head(const, gain, w, 0.0), (gain @ w)[None]) < 1e-12


def test_greedy_is_first_argmax():
    rng = np.random.default_rng(2)
    lg = rng.standard_normal((4, 5, 33))
    assert np.array_equal(gen.greedy(lg), np.argmax(lg, axis=-1))
    tie = np.zeros((1, 6))
    tie[0, 2] = tie[0, 4] = 7.0
    assert gen.greedy(tie)[0] == 2
    assert gen.greedy(-np.ones((1, 3)))[0] == 0


def _generate(w, n_new, prompt, head, wiring="ladder"):
    layers, cfg = helpers.oracle_model(w)
    state = lo.State.empty(cfg, w.n_real_shards, w.batch, prompt.shape[1] + n_new)
    toks, logits = gen.generate(prompt, n_new, head["table"], head["final_norm"], head["w_lm"], layers, cfg, state,
                                wiring=wiring)
    return toks, logits, layers, cfg


@pytest.mark.parametrize("wiring", ["ladder", "standard"])
def test_cached_generation_equals_full_recompute(wiring):
    """Every sampled position recomputed from scratch: the whole sequence so far through a fresh
    cache, head on its last position."""
    w = TINY.with_(name="tiny_gen", batch=2, prefill=5)
    head = _head(w)
    prompt = inputs.prompt_tokens(w.batch, w.prefill, VOCAB).numpy()
    n_new = 4
    toks, logits, layers, cfg = _generate(w, n_new, prompt, head, wiring)
    assert toks.shape == (2, n_new) and toks.min() >= 0 and toks.max() < VOCAB
    seq = prompt
    for i in range(n_new):
        state = lo.State.empty(cfg, w.n_real_shards, w.batch, seq.shape[1])
        x = lo.forward_eq2(gen.embed(seq, head["table"]), layers, cfg, state, wiring=wiring)
        full = gen.lm_head(x[:, -1], head["final_norm"], head["w_lm"], cfg.rms_eps)
        assert helpers.rel_err(logits[i], full) < 1e-9
        assert np.array_equal(np.argmax(full, axis=-1), toks[:, i])
        seq = np.concatenate([seq, toks[:, i:i + 1]], axis=1)


def test_generation_feeds_the_sampled_token_back():
    """Changing one prompt token of one sequence changes that sequence's continuation inputs only."""
    w = TINY.with_(name="tiny_gen", batch=2, prefill=4)
    head = _head(w)
    prompt = inputs.prompt_tokens(w.batch, w.prefill, VOCAB).numpy()
    a, la, _, _ = _generate(w, 3, prompt, head)
    other = prompt.copy()
    other[1, 0] = (other[1, 0] + 1) % VOCAB
    b, lb, _, _ = _generate(w, 3, other, head)
    assert np.array_equal(a[0], b[0]) and all(np.array_equal(x[0], y[0]) for x, y in zip(la, lb))
    assert not np.allclose(la[0][1], lb[0][1])


# ---- planted mistakes -----------------------------------------------------------------------------
def _pins_fail() -> bool:
    for f in (test_embed_is_a_row_gather_like_torch_embedding,
              test_lm_head_is_rms_norm_then_matmul_and_splits_over_the_vocabulary, test_greedy_is_first_argmax,
              lambda: test_cached_generation_equals_full_recompute("ladder"),
              test_generation_feeds_the_sampled_token_back):
        try:
            f()
        except Exception:
            return True
    return False


def test_planted_mistakes_in_the_generation_oracle_are_caught(monkeypatch):
    assert not _pins_fail()
    orig_embed, orig_head, orig_greedy, orig_generate = gen.embed, gen.lm_head, gen.greedy, gen.generate
    mutants = {
        "embed_off_by_one": ("embed", lambda tok, table: orig_embed((np.asarray(tok) + 1) % table.shape[0], table)),
        "embed_column": ("embed", lambda tok, table: orig_embed(tok, table)[..., ::-1]),
        "head_without_norm": ("lm_head", lambda x, g, w, eps: np.asarray(x) @ w),
        "head_without_gain": ("lm_head", lambda x, g, w, eps: orig_head(x, np.ones_like(g), w, eps)),
        "head_transposed": ("lm_head", lambda x, g, w, eps: orig_head(x, g, w[:, ::-1], eps)),
        "greedy_last_max": ("greedy", lambda lg: lg.shape[-1] - 1 - np.argmax(lg[..., ::-1], axis=-1)),
        "greedy_min": ("greedy", lambda lg: np.argmin(lg, axis=-1)),
    }
    for name, (attr, fn) in mutants.items():
        monkeypatch.setattr(gen, attr, fn)
        assert _pins_fail(), f"planted mistake {name} was not caught"
        monkeypatch.setattr(gen, attr, {"embed": orig_embed, "lm_head": orig_head, "greedy": orig_greedy}[attr])

    def stale_generate(prompt, n_new, table, gain, w_lm, layers, cfg, state, *a, **k):
        toks, lg = orig_generate(prompt, n_new, table, gain, w_lm, layers, cfg, state, *a, **k)
        return np.repeat(toks[:, :1], n_new, axis=1), lg       # never feeds the new token back
    monkeypatch.setattr(gen, "generate", stale_generate)
    assert _pins_fail(), "a loop that does not feed the sampled token back was not caught"
