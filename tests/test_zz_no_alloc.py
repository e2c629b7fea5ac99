"""The entry point that allocates nothing (ladder_head_static) against the entry point it is a variant of
(ladder_head), through the C-ABI: same greedy tokens, bit for bit, on two calls in a row, the second with a
smaller input (the static scratch keeps the first call's contents); limits are rejected with an error code."""
import ctypes as C

import pytest
import torch

from paper_2501_06589_amd import inputs, ladder

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TINY = inputs.WORKLOADS["tiny"]
SMALL_BF16 = TINY.with_(name="small_bf16_static", dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                        inter=352, tp_degree=1, n_real_shards=1, batch=5, prefill=8, decode_steps=1)


@pytest.mark.parametrize("w,vocab,vocab_local", [(SMALL_BF16, 1024, 512), (TINY.with_(name="tiny_static", batch=5), 300, None)])
def test_head_static_matches_head_on_two_calls_in_a_row(w, vocab, vocab_local):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lib = ladder.lib()
    ctx = ladder.Ladder(ladder.config_for(w))
    head = inputs.head_weights(w, vocab, vocab_local)
    ctx.load_head(*(head[k].to(DEV) for k in ("table", "final_norm", "w_lm")))
    g = torch.Generator().manual_seed(7)
    xs = [torch.randn((5, w.hidden), generator=g).to(DEV), torch.randn((2, w.hidden), generator=g).to(DEV)]
    for x in xs:                                   # 5 rows, then 2 rows over the same scratch
        rows = x.shape[0]
        _, want = ctx.head(x, want_logits=True)
        got = torch.full((rows,), -1, dtype=torch.int32, device=DEV)
        rc = lib.ladder_head_static(ctx._h, C.c_void_p(x.data_ptr()), rows, C.c_void_p(got.data_ptr()))
        assert rc == ladder.LADDER_OK, lib.ladder_last_error(ctx._h)
        torch.cuda.synchronize()
        assert torch.equal(got.cpu(), want.cpu()), (got.cpu().tolist(), want.cpu().tolist())
    # limits and misuse come back as error codes, with nothing launched
    got = torch.zeros((5,), dtype=torch.int32, device=DEV)
    assert lib.ladder_head_static(ctx._h, None, 5, C.c_void_p(got.data_ptr())) == ladder.LADDER_E_ARG
    assert lib.ladder_head_static(ctx._h, C.c_void_p(xs[0].data_ptr()), 6, C.c_void_p(got.data_ptr())) == ladder.LADDER_E_SHAPE
    ctx.free()


def test_head_static_rejects_sizes_beyond_its_scratch():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lib = ladder.lib()
    w = TINY.with_(name="tiny_static_big", batch=2)
    ctx = ladder.Ladder(ladder.config_for(w))
    vocab = 32768 + 64                              # vocab_local beyond LADDER_HEAD_STATIC_MAX_VOCAB
    head = inputs.head_weights(w, vocab, None)
    ctx.load_head(*(head[k].to(DEV) for k in ("table", "final_norm", "w_lm")))
    x = torch.randn((2, w.hidden)).to(DEV)
    got = torch.zeros((2,), dtype=torch.int32, device=DEV)
    assert lib.ladder_head_static(ctx._h, C.c_void_p(x.data_ptr()), 2, C.c_void_p(got.data_ptr())) == ladder.LADDER_E_SHAPE
    assert b"LADDER_HEAD_STATIC_MAX" in lib.ladder_last_error(ctx._h)
    _, want = ctx.head(x)                           # the allocating entry point still serves that size
    assert want.shape == (2,)
    ctx.free()
