"""The pins must bite: each planted mistake in the oracle (CPU only, patched in
place and restored) has to make at least one pin of test_oracle_pins fail."""
import numpy as np
import pytest

from oracle import ladder_oracle as lo
import test_oracle_pins as pins

PIN_FUNCS = [
    pins.test_rmsnorm_matches_torch_rms_norm, pins.test_rmsnorm_constant_vector_closed_form,
    pins.test_silu_matches_torch, pins.test_rope_is_complex_multiplication, pins.test_rope_invariants,
    lambda: pins.test_attention_matches_torch_sdpa(0), lambda: pins.test_attention_matches_torch_sdpa(5),
    pins.test_attention_special_cases, pins.test_round_bf16_matches_torch_cast,
    pins.test_mlp_matches_torch_and_gate_zero, pins.test_single_layer_closed_form,
    pins.test_two_layer_ladder_and_standard_against_torch_modules, pins.test_shard_sum_equals_unsharded,
    pins.test_eq2_form_equals_alg1_form, pins.test_ladder_reduces_to_standard_when_in_between_outputs_vanish,
    pins.test_kv_cached_decode_equals_full_recompute, pins.test_module_input_is_two_modules_stale,
    pins.test_causality_and_batch_independence, pins.test_reduce_is_linear_in_peer_partials,
    lambda: pins.test_brute_force_tiny(2, 2), pins.test_pipeline_stage_hands_over_the_index_forms_tensors,
]


def some_pin_fails() -> bool:
    for f in PIN_FUNCS:
        try:
            f()
        except AssertionError:
            return True
        except Exception:
            return True
    return False


def m_rope_sign(v, positions, theta):
    return _orig["rope"](v, -np.asarray(positions), theta)


def m_rope_halfsplit(v, positions, theta):
    d = v.shape[-1]
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])
    inv = np.argsort(perm)
    return _orig["rope"](v[..., inv], positions, theta)[..., perm]


def m_rope_freq(v, positions, theta):
    return _orig["rope"](v, positions, theta * 2)


def m_norm_eps_outside(x, gain, eps):
    return x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps) * gain


def m_norm_no_gain(x, gain, eps):
    return _orig["rmsnorm"](x, np.ones_like(gain), eps)


def m_norm_mean_subtracted(x, gain, eps):
    return _orig["rmsnorm"](x - x.mean(axis=-1, keepdims=True), gain, eps)


def m_silu_sigmoid_only(z):
    return 1.0 / (1.0 + np.exp(-z))


def m_attn_no_scale(q, k, v, s0):
    return _orig["causal_gqa_attention"](q * np.sqrt(q.shape[-1]), k, v, s0)


def m_attn_not_causal(q, k, v, s0):
    t = q.shape[1]
    return np.concatenate([_orig["causal_gqa_attention"](q[:, i:i + 1], k, v, s0 + t - 1) for i in range(t)], axis=1)


def m_attn_head_map(q, k, v, s0):
    nq, nkv = q.shape[2], k.shape[1]
    order = [(h % nkv) * (nq // nkv) + h // nkv for h in range(nq)]     # h -> h % nkv instead of h // group
    out = _orig["causal_gqa_attention"](q[:, :, np.argsort(order)], k, v, s0)
    return out[:, :, order]


def m_mlp_swapped(y, sh):
    return (lo.silu(y @ sh.w_up) * (y @ sh.w_gate)) @ sh.w_down


def m_allreduce_drop_peer(m, parts, peers, cfg):
    return _orig["all_reduce"](m, parts, None if peers is None else peers[:, :-1], cfg)


def m_allreduce_pool_shift(m, parts, peers, cfg):
    return _orig["all_reduce"](m + 1, parts, peers, cfg)


def m_allreduce_first_only(m, parts, peers, cfg):
    return _orig["all_reduce"](m, parts[:1], peers, cfg)


def m_lags_three(n, wiring):
    base = _orig["_lags"](n, wiring)
    return [3 if v == 2 else v for v in base]


def m_lags_parallel_as_ladder(n_modules, wiring):
    """The parallel attention / MLP block wired like the ladder."""
    return _orig["_lags"](n_modules, "ladder" if wiring == "parallel" else wiring)


def m_lags_parallel_swapped(n_modules, wiring):
    """Attention reads the stale stream and the MLP the fresh one instead of the other way round."""
    if wiring == "parallel":
        return [2 if m % 2 == 1 else 1 for m in range(1, n_modules + 1)]
    return _orig["_lags"](n_modules, wiring)


def m_round_truncate(a):
    m, e = np.frexp(np.asarray(a, dtype=np.float64))
    return np.ldexp(np.trunc(m * 256.0) / 256.0, e)


def m_stage_outputs_swapped(residual, attn_out, mlp_out, *a, **k):
    r, x, y = _orig["stage_alg1"](residual, attn_out, mlp_out, *a, **k)
    return r, y, x


def m_stage_inputs_swapped(residual, attn_out, mlp_out, *a, **k):
    return _orig["stage_alg1"](residual, mlp_out, attn_out, *a, **k)


def m_stage_drops_handed_over_mlp(residual, attn_out, mlp_out, *a, **k):
    return _orig["stage_alg1"](residual, attn_out, None, *a, **k)


def m_stage_residual_complete(residual, attn_out, mlp_out, *a, **k):
    r, x, y = _orig["stage_alg1"](residual, attn_out, mlp_out, *a, **k)
    return r + x, x, y          # hands over the stream with the attention output already in it, and the output again


def m_stage_ignores_module_offset(residual, attn_out, mlp_out, layers, cfg, state=None, peers=None, module_offset=0):
    return _orig["stage_alg1"](residual, attn_out, mlp_out, layers, cfg, state, peers, 1 if module_offset else 0)


MUTANTS = {
    "rope": [m_rope_sign, m_rope_halfsplit, m_rope_freq],
    "rmsnorm": [m_norm_eps_outside, m_norm_no_gain, m_norm_mean_subtracted],
    "silu": [m_silu_sigmoid_only],
    "causal_gqa_attention": [m_attn_no_scale, m_attn_not_causal, m_attn_head_map],
    "mlp_partial": [m_mlp_swapped],
    "all_reduce": [m_allreduce_drop_peer, m_allreduce_pool_shift, m_allreduce_first_only],
    "_lags": [m_lags_three, m_lags_parallel_as_ladder, m_lags_parallel_swapped],
    "round_bf16": [m_round_truncate],
    "stage_alg1": [m_stage_outputs_swapped, m_stage_inputs_swapped, m_stage_drops_handed_over_mlp, m_stage_residual_complete,
                   m_stage_ignores_module_offset],
}
_orig = {k: getattr(lo, k) for k in MUTANTS}


def test_pins_pass_unmutated():
    assert not some_pin_fails()


@pytest.mark.parametrize("name,mutant", [(k, f) for k, fs in MUTANTS.items() for f in fs],
                         ids=lambda v: v if isinstance(v, str) else v.__name__)
def test_planted_mistake_is_caught(name, mutant, monkeypatch):
    monkeypatch.setattr(lo, name, mutant)
    assert some_pin_fails(), f"no pin notices {mutant.__name__}"
