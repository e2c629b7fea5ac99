"""Pins of the CPU oracle against things other than itself (CPU only).

Each test cites what fixes the expected value: the paper's identities (TP sharding
rule, Eq. 1 vs Eq. 2, Algorithm 1), closed forms, invariants, torch float64
library routines, or brute force with python loops written here independently.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ladder_oracle as lo

RNG = np.random.default_rng(1234)


def rand_model(n_layers=2, hidden=16, nq=2, nkv=1, d=4, inter=6, n_shards=2, storage="exact", theta=100.0,
               rng=None):
    rng = rng or np.random.default_rng(7)
    cfg = lo.OracleConfig(n_layers, hidden, nq, nkv, d, inter, 1e-5, theta, storage, 1)
    layers = []
    for _ in range(n_layers):
        shards = [lo.ShardLayer(rng.normal(0, 0.3, (hidden, nq * d)), rng.normal(0, 0.3, (hidden, nkv * d)),
                                rng.normal(0, 0.3, (hidden, nkv * d)), rng.normal(0, 0.3, (nq * d, hidden)),
                                rng.normal(0, 0.3, (hidden, inter)), rng.normal(0, 0.3, (hidden, inter)),
                                rng.normal(0, 0.3, (inter, hidden))) for _ in range(n_shards)]
        layers.append(lo.Layer(1 + 0.1 * rng.normal(size=hidden), 1 + 0.1 * rng.normal(size=hidden), shards))
    return layers, cfg


def rms(a):
    return float(np.sqrt(np.mean(np.square(a))))


# --------------------------------------------------------------------------- op level vs library routines
def test_rmsnorm_matches_torch_rms_norm():
    x = RNG.normal(size=(3, 5, 32)) * 3
    g = 1 + 0.1 * RNG.normal(size=32)
    want = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.max(np.abs(lo.rmsnorm(x, g, 1e-5) - want)) < 1e-12


def test_rmsnorm_constant_vector_closed_form():
    # constant vector c, unit gain: c / sqrt(c^2 + eps)
    for c in (2.5, -0.3):
        y = lo.rmsnorm(np.full((1, 8), c), np.ones(8), 1e-5)
        assert np.allclose(y, c / math.sqrt(c * c + 1e-5), atol=1e-14)
    # eps sits inside the square root: for x = 0 the output is 0, not inf/nan
    assert np.all(lo.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-5) == 0)


def test_silu_matches_torch():
    z = RNG.normal(size=1000) * 4
    assert np.max(np.abs(lo.silu(z) - F.silu(torch.from_numpy(z)).numpy())) < 1e-14


def test_rope_is_complex_multiplication():
    # pair (v[2j], v[2j+1]) as a complex number times exp(i * pos * theta^(-2j/d))
    t_sz, nh, d, theta = 6, 3, 8, 500.0
    v = RNG.normal(size=(2, t_sz, nh, d))
    pos = np.array([0, 1, 2, 7, 100, 2047])
    z = torch.view_as_complex(torch.from_numpy(v).reshape(2, t_sz, nh, d // 2, 2).contiguous())
    ang = torch.tensor(pos, dtype=torch.float64)[:, None] * theta ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    want = torch.view_as_real(z * torch.polar(torch.ones_like(ang), ang)[None, :, None, :]).reshape(2, t_sz, nh, d)
    assert np.max(np.abs(lo.rope(v, pos, theta) - want.numpy())) < 1e-12


def test_rope_invariants():
    d, theta = 16, 1e4
    q = RNG.normal(size=(1, 1, 1, d))
    k = RNG.normal(size=(1, 1, 1, d))
    # position 0 is the identity
    assert np.array_equal(lo.rope(q, [0], theta), q)
    # norm preserving
    assert abs(np.linalg.norm(lo.rope(q, [37], theta)) - np.linalg.norm(q)) < 1e-12
    # <rope(q,a), rope(k,b)> depends on a - b only
    dots = [float(np.sum(lo.rope(q, [a], theta) * lo.rope(k, [a - 5], theta))) for a in (5, 9, 300)]
    assert max(dots) - min(dots) < 1e-10
    # first pair turns by exactly pos radians (theta^0 = 1), last pair by pos * theta^(-(d-2)/d)
    e0 = np.zeros((1, 1, 1, d)); e0[..., 0] = 1.0
    r = lo.rope(e0, [2], theta)
    assert abs(r[0, 0, 0, 0] - math.cos(2.0)) < 1e-14 and abs(r[0, 0, 0, 1] - math.sin(2.0)) < 1e-14
    el = np.zeros((1, 1, 1, d)); el[..., d - 2] = 1.0
    r = lo.rope(el, [3], theta)
    a = 3 * theta ** (-(d - 2) / d)
    assert abs(r[0, 0, 0, d - 2] - math.cos(a)) < 1e-14 and abs(r[0, 0, 0, d - 1] - math.sin(a)) < 1e-14


@pytest.mark.parametrize("s0", [0, 5])
def test_attention_matches_torch_sdpa(s0):
    b, t, nq, nkv, d = 2, 7, 4, 2, 8
    q = RNG.normal(size=(b, t, nq, d))
    k = RNG.normal(size=(b, nkv, s0 + t, d))
    v = RNG.normal(size=(b, nkv, s0 + t, d))
    got = lo.causal_gqa_attention(q, k, v, s0)
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)                       # [B, nq, T, d]
    tk = torch.from_numpy(k).repeat_interleave(nq // nkv, dim=1)       # kv head of q head h is h // group
    tv = torch.from_numpy(v).repeat_interleave(nq // nkv, dim=1)
    mask = torch.arange(s0 + t)[None, :] <= (s0 + torch.arange(t))[:, None]
    want = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask).permute(0, 2, 1, 3).numpy()
    assert np.max(np.abs(got - want)) < 1e-12


def test_attention_special_cases():
    b, nq, nkv, d = 1, 2, 1, 4
    k = RNG.normal(size=(b, nkv, 6, d))
    v = RNG.normal(size=(b, nkv, 6, d))
    # a single visible position returns its value vector
    q = RNG.normal(size=(b, 1, nq, d))
    out = lo.causal_gqa_attention(q, k, v, 0)
    assert np.allclose(out[0, 0, 0], v[0, 0, 0]) and np.allclose(out[0, 0, 1], v[0, 0, 0])
    # q = 0: uniform weights -> causal running mean of V
    out = lo.causal_gqa_attention(np.zeros((b, 6, nq, d)), k, v, 0)
    want = np.cumsum(v[0, 0], axis=0) / np.arange(1, 7)[:, None]
    assert np.allclose(out[0, :, 0], want, atol=1e-14)
    # one dominating key: a huge score puts all the weight on it (softmax, not a plain normalisation)
    k2 = np.zeros((1, 1, 3, d)); k2[0, 0, 1, 0] = 1.0
    q2 = np.zeros((1, 1, 1, d)); q2[..., 0] = 1e3
    out = lo.causal_gqa_attention(q2, k2, v[:, :, :3], 2)
    assert np.allclose(out[0, 0, 0], v[0, 0, 1], atol=1e-12)
    # scale is 1/sqrt(d): two keys with q.k = sqrt(d)*ln(3) and 0 get weights 3/4 and 1/4
    k3 = np.zeros((1, 1, 2, d)); k3[0, 0, 0, 0] = 1.0
    q3 = np.zeros((1, 1, 1, d)); q3[..., 0] = math.sqrt(d) * math.log(3.0)
    v3 = np.zeros((1, 1, 2, d)); v3[0, 0, 0, 0] = 1.0; v3[0, 0, 1, 1] = 1.0
    out = lo.causal_gqa_attention(q3, k3, v3, 1)
    assert np.allclose(out[0, 0, 0, :2], [0.75, 0.25], atol=1e-14)


def test_round_bf16_matches_torch_cast():
    x = np.concatenate([RNG.normal(size=5000) * 3, RNG.normal(size=2000) * 1e-3, [1.00390625, 1.01171875, 0.0, -2.0]])
    x32 = x.astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).double().numpy()
    assert np.array_equal(lo.round_bf16(x32.astype(np.float64)), want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert lo.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert lo.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6


def test_mlp_matches_torch_and_gate_zero():
    layers, cfg = rand_model()
    sh = layers[0].shards[0]
    y = RNG.normal(size=(2, 3, cfg.hidden))
    ty = torch.from_numpy(y)
    want = (F.silu(ty @ torch.from_numpy(sh.w_gate)) * (ty @ torch.from_numpy(sh.w_up))) @ torch.from_numpy(sh.w_down)
    assert np.max(np.abs(lo.mlp_partial(y, sh) - want.numpy())) < 1e-12
    zero_gate = lo.ShardLayer(sh.wq, sh.wk, sh.wv, sh.wo, np.zeros_like(sh.w_gate), sh.w_up, sh.w_down)
    assert np.all(lo.mlp_partial(y, zero_gate) == 0)


# --------------------------------------------------------------------------- model level
def torch_attention_module(x, gain, sh, cfg, theta):
    """Independent attention module (unsharded weights) built from torch float64 routines."""
    b, t, h = x.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    tx = torch.from_numpy(x)
    y = F.rms_norm(tx, (h,), torch.from_numpy(gain), eps=cfg.rms_eps)

    def rot(z, n):  # rotary by complex multiplication
        zc = torch.view_as_complex(z.reshape(b, t, n, d // 2, 2).contiguous())
        ang = torch.arange(t, dtype=torch.float64)[:, None] * theta ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
        return torch.view_as_real(zc * torch.polar(torch.ones_like(ang), ang)[None, :, None, :]).reshape(b, t, n, d)

    q = rot(y @ torch.from_numpy(sh.wq), nq).permute(0, 2, 1, 3)
    k = rot(y @ torch.from_numpy(sh.wk), nkv).permute(0, 2, 1, 3).repeat_interleave(nq // nkv, dim=1)
    v = (y @ torch.from_numpy(sh.wv)).reshape(b, t, nkv, d).permute(0, 2, 1, 3).repeat_interleave(nq // nkv, dim=1)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(b, t, nq * d)
    return (o @ torch.from_numpy(sh.wo)).numpy()


def torch_mlp_module(x, gain, sh, cfg):
    tx = torch.from_numpy(x)
    y = F.rms_norm(tx, (x.shape[-1],), torch.from_numpy(gain), eps=cfg.rms_eps)
    return ((F.silu(y @ torch.from_numpy(sh.w_gate)) * (y @ torch.from_numpy(sh.w_up))) @ torch.from_numpy(sh.w_down)).numpy()


def test_single_layer_closed_form():
    """N = 1: both modules read x_0, so x_2 = E + Attn(norm_a(E)) + MLP(norm_m(E))
    (the parallel attention+MLP block), built here from torch routines."""
    layers, cfg = rand_model(n_layers=1, n_shards=1, nq=4, nkv=2, d=8, hidden=32, inter=12)
    emb = RNG.normal(size=(2, 5, cfg.hidden))
    want = emb + torch_attention_module(emb, layers[0].attn_norm, layers[0].shards[0], cfg, cfg.rope_theta) \
        + torch_mlp_module(emb, layers[0].mlp_norm, layers[0].shards[0], cfg)
    for fwd in (lo.forward_eq2, lo.forward_alg1):
        assert np.max(np.abs(fwd(emb, layers, cfg) - want)) < 1e-11


def test_two_layer_ladder_and_standard_against_torch_modules():
    """N = 2, written out by hand from Eq. 2 and Eq. 1 with the torch modules."""
    layers, cfg = rand_model(n_layers=2, n_shards=1, nq=4, nkv=2, d=8, hidden=32, inter=12)
    emb = RNG.normal(size=(1, 6, cfg.hidden))
    A = lambda i, x: torch_attention_module(x, layers[i].attn_norm, layers[i].shards[0], cfg, cfg.rope_theta)
    M = lambda i, x: torch_mlp_module(x, layers[i].mlp_norm, layers[i].shards[0], cfg)
    # ladder: h1(x0), h2(x0), h3(x1), h4(x2)
    x0 = emb; x1 = x0 + A(0, x0); x2 = x1 + M(0, x0); x3 = x2 + A(1, x1); x4 = x3 + M(1, x2)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg) - x4)) < 1e-11
    assert np.max(np.abs(lo.forward_alg1(emb, layers, cfg) - x4)) < 1e-11
    # standard: h_m(x_{m-1})
    s1 = x0 + A(0, x0); s2 = s1 + M(0, s1); s3 = s2 + A(1, s2); s4 = s3 + M(1, s3)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg, wiring="standard") - s4)) < 1e-11
    assert np.max(np.abs(x4 - s4)) > 1e-3          # the two wirings are different functions
    # hybrid: layer 1 standard, layer 2 ladder -> h3 reads x1, h4 reads x2 of the standard prefix
    y3 = s2 + A(1, s1); y4 = y3 + M(1, s2)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg, wiring=[1, 1, 2, 2]) - y4)) < 1e-11
    # parallel attention / MLP block: layer output = layer input + A(layer input) + M(layer input)
    p2 = x0 + A(0, x0) + M(0, x0); p4 = p2 + A(1, p2) + M(1, p2)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg, wiring="parallel") - p4)) < 1e-11
    assert np.max(np.abs(p4 - s4)) > 1e-3 and np.max(np.abs(p4 - x4)) > 1e-3


def test_shard_sum_equals_unsharded():
    """(XA)B = sum_r (X A_r) B_r: R shards summed == the merged single-rank model."""
    for r in (2, 4):
        layers, cfg = rand_model(n_layers=3, n_shards=r, nq=2, nkv=1)
        merged, full_cfg = lo.merge_shards(layers, cfg)
        emb = RNG.normal(size=(2, 6, cfg.hidden))
        a = lo.forward_eq2(emb, layers, cfg)
        b = lo.forward_eq2(emb, merged, full_cfg)
        assert np.max(np.abs(a - b)) < 1e-10 * max(1.0, rms(b))
        # module level too
        u = RNG.normal(size=(1, 4, cfg.hidden))
        for m in (1, 2):
            assert np.max(np.abs(sum(lo.module_partials(m, u, layers, cfg, None, 0))
                                 - lo.module_partials(m, u, merged, full_cfg, None, 0)[0])) < 1e-11


def test_eq2_form_equals_alg1_form():
    layers, cfg = rand_model(n_layers=4, n_shards=2)
    emb = RNG.normal(size=(2, 5, cfg.hidden))
    peers = RNG.normal(size=(3, 2, 10, cfg.hidden)) * 0.1
    a = lo.forward_eq2(emb, layers, cfg, peers=peers)
    b = lo.forward_alg1(emb, layers, cfg, peers=peers)
    assert np.max(np.abs(a - b)) < 1e-12
    # with caches and a later decode call as well
    sa = lo.State.empty(cfg, 2, 2, 8); sb = lo.State.empty(cfg, 2, 2, 8)
    lo.forward_eq2(emb, layers, cfg, sa); lo.forward_alg1(emb, layers, cfg, sb)
    e2 = RNG.normal(size=(2, 1, cfg.hidden))
    assert np.max(np.abs(lo.forward_eq2(e2, layers, cfg, sa) - lo.forward_alg1(e2, layers, cfg, sb))) < 1e-12
    assert sa.pos == sb.pos == 6


def test_pipeline_stage_hands_over_the_index_forms_tensors():
    """Section "Compatibility with other Parallelism Techniques": what a stage returns is the stream without
    the last two module outputs and those two outputs, each by itself (a swap or a dropped term fails), and a
    model cut into stages is the same model."""
    layers, cfg = rand_model(n_layers=5, n_shards=2)
    emb = RNG.normal(size=(2, 4, cfg.hidden))
    peers = RNG.normal(size=(4, 2, 8, cfg.hidden)) * 0.1
    trace = {}
    full = lo.forward_eq2(emb, layers, cfg, peers=peers, trace=trace)
    n_mod = 2 * cfg.n_layers
    r, a, m = lo.stage_alg1(emb, None, None, layers, cfg, peers=peers)
    assert np.max(np.abs(r - trace["x"][n_mod - 2])) < 1e-12
    assert np.max(np.abs(a - trace["h"][n_mod - 1])) < 1e-12
    assert np.max(np.abs(m - trace["h"][n_mod])) < 1e-12
    assert np.max(np.abs(r + a + m - full)) < 1e-12
    assert np.max(np.abs(a - m)) > 1e-3            # (the two outputs are not interchangeable)
    # cut after 2 and after 3 layers, with caches, prefill then one decode step
    import dataclasses
    cuts = [(0, 2), (2, 3), (3, 5)]
    whole = lo.State.empty(cfg, 2, 2, 8)
    stages = [(layers[i:j], dataclasses.replace(cfg, n_layers=j - i), lo.State.empty(dataclasses.replace(cfg, n_layers=j - i), 2, 2, 8), 2 * i)
              for i, j in cuts]
    for x in (emb, RNG.normal(size=(2, 1, cfg.hidden))):
        want = lo.stage_alg1(x, None, None, layers, cfg, whole, peers)
        got = (x, None, None)
        for ly, scfg, st, off in stages:
            got = lo.stage_alg1(*got, ly, scfg, st, peers, module_offset=off)
        for w, g_ in zip(want, got):
            assert np.max(np.abs(w - g_)) < 1e-12
    assert whole.pos == 5 and all(st.pos == 5 for _, _, st, _ in stages)
    # the intermediate hand-off matters: feeding a later stage the summed stream instead is another function
    mid = lo.stage_alg1(emb, None, None, layers[:2], stages[0][1], None, peers)
    merged = lo.stage_alg1(mid[0] + mid[1] + mid[2], None, None, layers[2:], dataclasses.replace(cfg, n_layers=3), None, peers, 4)
    split = lo.stage_alg1(*mid, layers[2:], dataclasses.replace(cfg, n_layers=3), None, peers, 4)
    assert np.max(np.abs(sum(merged) - sum(split))) > 1e-3
    assert np.max(np.abs(sum(split) - full)) < 1e-12


def zero_field(layers, name):
    out = []
    for ly in layers:
        shards = []
        for s in ly.shards:
            kw = {k: getattr(s, k) for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")}
            for n in name:
                kw[n] = np.zeros_like(kw[n])
            shards.append(lo.ShardLayer(**kw))
        out.append(lo.Layer(ly.attn_norm, ly.mlp_norm, shards))
    return out


def test_ladder_reduces_to_standard_when_in_between_outputs_vanish():
    """If every attention module outputs zero then x_{m-1} = x_{m-2} for even m, and odd
    modules' outputs are zero anyway, so Eq. 2 and Eq. 1 give the same x_2N; same with MLPs zeroed."""
    layers, cfg = rand_model(n_layers=3, n_shards=2)
    emb = RNG.normal(size=(1, 5, cfg.hidden))
    for fields in (("wo",), ("w_down",)):
        z = zero_field(layers, fields)
        a = lo.forward_eq2(emb, z, cfg, wiring="ladder")
        b = lo.forward_eq2(emb, z, cfg, wiring="standard")
        assert np.max(np.abs(a - b)) < 1e-12
        assert np.max(np.abs(a - emb)) > 1e-3
    z = zero_field(layers, ("wo", "w_down"))
    assert np.array_equal(lo.forward_eq2(emb, z, cfg), emb)


def test_kv_cached_decode_equals_full_recompute():
    for storage in ("exact", "bf16"):
        layers, cfg = rand_model(n_layers=3, n_shards=2, storage=storage)
        p, k = 5, 3
        emb = RNG.normal(size=(2, p + k, cfg.hidden))
        full = lo.forward_eq2(emb, layers, cfg)                        # no cache at all
        st = lo.State.empty(cfg, 2, 2, p + k)
        out = lo.forward_eq2(emb[:, :p], layers, cfg, st)
        assert np.max(np.abs(out - full[:, :p])) < 1e-11
        for i in range(k):
            out = lo.forward_eq2(emb[:, p + i:p + i + 1], layers, cfg, st)
            assert np.max(np.abs(out[:, 0] - full[:, p + i])) < 1e-11
        assert st.pos == p + k


def test_module_input_is_two_modules_stale():
    """Module m reads x_{m-2}: changing module m-1 leaves its input untouched, changing
    module m-2 does not."""
    layers, cfg = rand_model(n_layers=3, n_shards=1)
    emb = RNG.normal(size=(1, 4, cfg.hidden))
    base = {}
    lo.forward_eq2(emb, layers, cfg, trace=base)

    def perturbed(module):
        li, is_attn = (module - 1) // 2, module % 2 == 1
        out = list(layers)
        s = layers[li].shards[0]
        kw = {k: getattr(s, k) for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")}
        key = "wo" if is_attn else "w_down"
        kw[key] = kw[key] * 1.5
        out[li] = lo.Layer(layers[li].attn_norm, layers[li].mlp_norm, [lo.ShardLayer(**kw)])
        tr = {}
        lo.forward_eq2(emb, out, cfg, trace=tr)
        return tr

    for m in range(3, 7):
        assert np.array_equal(perturbed(m - 1)["u"][m], base["u"][m])
        assert np.max(np.abs(perturbed(m - 2)["u"][m] - base["u"][m])) > 1e-6
        # while the residual stream itself does see module m-1
        assert np.max(np.abs(perturbed(m - 1)["x"][m - 1] - base["x"][m - 1])) > 1e-6
    # modules 1 and 2 both read x_0
    assert base["u"][1] is base["x"][0] and base["u"][2] is base["x"][0]


def test_causality_and_batch_independence():
    layers, cfg = rand_model(n_layers=2, n_shards=2)
    emb = RNG.normal(size=(2, 6, cfg.hidden))
    base = lo.forward_eq2(emb, layers, cfg)
    e2 = emb.copy(); e2[0, 4] += 1.0
    out = lo.forward_eq2(e2, layers, cfg)
    assert np.array_equal(out[0, :4], base[0, :4])          # earlier tokens unchanged
    assert np.array_equal(out[1], base[1])                  # other sequence unchanged
    assert np.max(np.abs(out[0, 4:] - base[0, 4:])) > 1e-6  # later ones do change


def test_reduce_is_linear_in_peer_partials():
    layers, cfg = rand_model(n_layers=2, n_shards=1)
    emb = RNG.normal(size=(2, 3, cfg.hidden))
    peers = RNG.normal(size=(2, 3, 6, cfg.hidden)) * 0.1       # pool 2, 3 peers, 6 rows
    tr = {}
    lo.forward_eq2(emb, layers, cfg, peers=peers, trace=tr)
    for m in range(1, 5):
        real = sum(lo.module_partials(m, tr["u"][m], layers, cfg, None, 0))
        want_peers = peers[m % 2].sum(axis=0).reshape(2, 3, cfg.hidden)
        assert np.max(np.abs(tr["x"][m] - tr["x"][m - 1] - real - want_peers)) < 1e-12


# --------------------------------------------------------------------------- brute force, python loops only
def brute_force_ladder(emb, layers, cfg, peers=None, lag=2):
    """Independent scalar-loop evaluation of the ladder stack (lists of floats, math module)."""
    bsz, tsz, hid = emb.shape
    nq, nkv, d, inter = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.inter
    grp = nq // nkv

    def norm(row, gain):
        ms = sum(v * v for v in row) / hid
        return [row[i] / math.sqrt(ms + cfg.rms_eps) * gain[i] for i in range(hid)]

    def vecmat(vec, w):   # vec [K], w [K][N]
        return [sum(vec[k] * w[k][n] for k in range(len(vec))) for n in range(len(w[0]))]

    def rotate(vec, pos):  # one head [d]
        out = list(vec)
        for j in range(d // 2):
            ang = pos * cfg.rope_theta ** (-2.0 * j / d)
            c, s = math.cos(ang), math.sin(ang)
            out[2 * j] = vec[2 * j] * c - vec[2 * j + 1] * s
            out[2 * j + 1] = vec[2 * j] * s + vec[2 * j + 1] * c
        return out

    xs = [[[list(map(float, emb[b, t])) for t in range(tsz)] for b in range(bsz)]]
    for m in range(1, 2 * cfg.n_layers + 1):
        ly = layers[(m - 1) // 2]
        u = xs[max(m - lag, 0)]
        new = [[None] * tsz for _ in range(bsz)]
        for b in range(bsz):
            h_rows = [[0.0] * hid for _ in range(tsz)]
            for sh in ly.shards:
                if m % 2 == 1:
                    ys = [norm(u[b][t], ly.attn_norm) for t in range(tsz)]
                    qs = [vecmat(y, sh.wq.tolist()) for y in ys]
                    ks = [vecmat(y, sh.wk.tolist()) for y in ys]
                    vs = [vecmat(y, sh.wv.tolist()) for y in ys]
                    for t in range(tsz):
                        o = []
                        for h in range(nq):
                            kvh = h // grp
                            qh = rotate(qs[t][h * d:(h + 1) * d], t)
                            sc = []
                            for j in range(t + 1):
                                kh = rotate(ks[j][kvh * d:(kvh + 1) * d], j)
                                sc.append(sum(qh[i] * kh[i] for i in range(d)) / math.sqrt(d))
                            mx = max(sc)
                            ex = [math.exp(s - mx) for s in sc]
                            z = sum(ex)
                            o += [sum(ex[j] / z * vs[j][kvh * d + i] for j in range(t + 1)) for i in range(d)]
                        p = vecmat(o, sh.wo.tolist())
                        h_rows[t] = [h_rows[t][i] + p[i] for i in range(hid)]
                else:
                    for t in range(tsz):
                        y = norm(u[b][t], ly.mlp_norm)
                        g = vecmat(y, sh.w_gate.tolist())
                        up = vecmat(y, sh.w_up.tolist())
                        a = [g[i] / (1.0 + math.exp(-g[i])) * up[i] for i in range(inter)]
                        p = vecmat(a, sh.w_down.tolist())
                        h_rows[t] = [h_rows[t][i] + p[i] for i in range(hid)]
            for t in range(tsz):
                extra = [0.0] * hid
                if peers is not None:
                    for j in range(peers.shape[1]):
                        extra = [extra[i] + float(peers[m % peers.shape[0], j, b * tsz + t, i]) for i in range(hid)]
                new[b][t] = [xs[m - 1][b][t][i] + h_rows[t][i] + extra[i] for i in range(hid)]
        xs.append(new)
    return np.array(xs[-1])


@pytest.mark.parametrize("n_layers,n_shards", [(1, 1), (2, 2)])
def test_brute_force_tiny(n_layers, n_shards):
    layers, cfg = rand_model(n_layers=n_layers, hidden=8, nq=2, nkv=1, d=4, inter=5, n_shards=n_shards)
    emb = RNG.normal(size=(2, 3, 8))
    peers = RNG.normal(size=(2, 2, 6, 8)) * 0.1
    want = brute_force_ladder(emb, layers, cfg, peers)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg, peers=peers) - want)) < 1e-11
    assert np.max(np.abs(lo.forward_alg1(emb, layers, cfg, peers=peers) - want)) < 1e-11
    want_std = brute_force_ladder(emb, layers, cfg, peers, lag=1)
    assert np.max(np.abs(lo.forward_eq2(emb, layers, cfg, peers=peers, wiring="standard") - want_std)) < 1e-11
