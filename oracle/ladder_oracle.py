"""CPU oracle for the Ladder-Residual shard forward.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the bench's ``cpu_baseline`` leg may
import this file; the product (the HIP library and its binding) never does,
and this file imports nothing from the product.  Everything is plain numpy in
float64, written for reading against the paper, not for speed: no blocking, no
fusion, no reordering beyond what the definitions state.

What it computes (paper: section "Ladder Transformer", Eq. 2; Algorithm 1;
section "Tensor Parallelism Background" for the sharding rule and Eq. 1):

  * one tensor-parallel rank's (or several ranks') partial sums of Llama-3
    style modules h_m -- odd m: RMSNorm -> q,k,v projections -> rotary
    embedding -> causal grouped-query attention over a KV cache -> output
    projection; even m: RMSNorm -> SwiGLU MLP;
  * the "AllReduce" as a plain sum over the partial sums of all ranks (the
    ranks that are not computed contribute given synthetic partials);
  * the ladder recurrence   x*_m = h_m(x_{m-2}),  x_m = AllReduce(x*_m) + x_{m-1}
    (Eq. 2), in an index form (`forward_eq2`) and in the variable-passing form
    of Algorithm 1 (`forward_alg1`), plus the standard wiring of Eq. 1 and a
    per-module mix of both (hybrid) through `src_lag`;
  * a pipeline stage (`stage_alg1`): a run of layers that takes and returns the
    three tensors Algorithm 1 passes from block to block (section "Compatibility
    with other Parallelism Techniques").

Readings where the paper is silent:
modules 1 and 2 both read x_0; after the last layer the two outstanding module
outputs are added (x_2N); RMSNorm with eps inside the square root; rotary
embedding on adjacent pairs (2j, 2j+1) with angle pos * theta^(-2j/d) and no
long-context rescaling; softmax scale 1/sqrt(d); q head h uses kv head
floor(h / (nq/nkv)); no biases.  Storage roundings are part of the problem
statement: in a bf16 workload the KV-cache entries are rounded to bf16 when
they are stored (weights, embeddings and peer partials arrive already rounded).

Pins (tests, CPU only): shard-sum == unsharded; ladder == standard when the
in-between module outputs are zero; cached decode == full recompute; Eq.-2
form == Algorithm-1 form; single-layer closed form; staleness of inputs;
a pipeline stage's three tensors == the index form's x_{2N-2}, h_{2N-1}, h_{2N},
and stages in a row == one stage; op-level agreement with torch float64 library routines; rotary / softmax /
norm invariants; causality; brute force with python loops on hand-sized
models.  The paper prints no numeric example, so no printed value pins it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# storage rounding
# ---------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (8 significant bits, ties to even); result kept as float64.
    Written from the format's definition; exponent range is not modelled (values
    here are far from bf16 overflow/underflow)."""
    a = np.asarray(a, dtype=F64)
    m, e = np.frexp(a)                      # a = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.round(m * 256.0) / 256.0, e)   # np.round: half to even


def round_storage(a: np.ndarray, storage: str) -> np.ndarray:
    if storage == "bf16":
        return round_bf16(a)
    if storage == "fp32":
        return np.asarray(a, dtype=np.float32).astype(F64)
    if storage == "exact":
        return np.asarray(a, dtype=F64)
    raise ValueError(storage)


# ---------------------------------------------------------------------------
# configuration, weights, state
# ---------------------------------------------------------------------------
@dataclass
class OracleConfig:
    """Sizes are LOCAL (per tensor-parallel shard)."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    inter: int
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    storage: str = "fp32"            # rounding applied to stored KV entries: fp32 | bf16 | exact
    peer_pool: int = 1


@dataclass
class ShardLayer:
    """One shard's slice of one layer; matrices are [in_features, out_features]."""
    wq: np.ndarray       # [H, nq*d]   columns of this shard's query heads
    wk: np.ndarray       # [H, nkv*d]
    wv: np.ndarray       # [H, nkv*d]
    wo: np.ndarray       # [nq*d, H]   rows of the same query heads
    w_gate: np.ndarray   # [H, I]
    w_up: np.ndarray     # [H, I]
    w_down: np.ndarray   # [I, H]


@dataclass
class Layer:
    attn_norm: np.ndarray            # [H] gain, replicated on every rank
    mlp_norm: np.ndarray             # [H]
    shards: List[ShardLayer]         # the ranks that are computed


@dataclass
class State:
    """KV cache of every (layer, shard) and the number of cached positions."""
    k: List[List[np.ndarray]]        # [layer][shard] -> [B, nkv, max_seq, d]
    v: List[List[np.ndarray]]
    pos: int = 0

    @staticmethod
    def empty(cfg: OracleConfig, n_shards: int, batch: int, max_seq: int) -> "State":
        shp = (batch, cfg.n_kv_heads, max_seq, cfg.head_dim)
        return State(k=[[np.zeros(shp, F64) for _ in range(n_shards)] for _ in range(cfg.n_layers)],
                     v=[[np.zeros(shp, F64) for _ in range(n_shards)] for _ in range(cfg.n_layers)],
                     pos=0)


# ---------------------------------------------------------------------------
# module pieces (Llama-3 style; the paper fixes only "Llama-3's model architecture")
# ---------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y_i = x_i * gain_i / sqrt(mean_k(x_k^2) + eps) over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(v: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding.  v: [..., T, n_heads, d]; positions: [T].
    Pair (v[2j], v[2j+1]) is rotated by the angle positions[t] * theta**(-2j/d)."""
    d = v.shape[-1]
    j = np.arange(d // 2, dtype=F64)
    inv_freq = theta ** (-2.0 * j / d)                                  # [d/2]
    ang = np.asarray(positions, dtype=F64)[:, None] * inv_freq[None, :]  # [T, d/2]
    cos = np.cos(ang)[:, None, :]                                        # [T, 1, d/2]
    sin = np.sin(ang)[:, None, :]
    even, odd = v[..., 0::2], v[..., 1::2]
    out = np.empty_like(v)
    out[..., 0::2] = even * cos - odd * sin
    out[..., 1::2] = even * sin + odd * cos
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def causal_gqa_attention(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, s0: int) -> np.ndarray:
    """q: [B, T, nq, d] for the T new positions s0 .. s0+T-1;
    k_all, v_all: [B, nkv, >= s0+T, d] holding every position 0 .. s0+T-1.
    Query t sees keys j <= s0 + t.  Returns [B, T, nq, d]."""
    b_sz, t_sz, nq, d = q.shape
    nkv = k_all.shape[1]
    group = nq // nkv
    out = np.zeros_like(q)
    for b in range(b_sz):
        for h in range(nq):
            kv = h // group
            for t in range(t_sz):
                n_vis = s0 + t + 1
                scores = k_all[b, kv, :n_vis] @ q[b, t, h] / np.sqrt(float(d))   # [n_vis]
                w = np.exp(scores - scores.max())
                w = w / w.sum()
                out[b, t, h] = w @ v_all[b, kv, :n_vis]
    return out


def attention_partial(y: np.ndarray, sh: ShardLayer, cfg: OracleConfig, s0: int,
                      cache_k: Optional[np.ndarray], cache_v: Optional[np.ndarray]) -> np.ndarray:
    """One shard's partial sum of the attention module on normed input y [B, T, H]
    for new positions s0 .. s0+T-1.  With a cache, the new k, v are appended to it
    (after storage rounding) and attention runs over the cache; without one
    (cache_k is None, s0 must be 0) it runs over this call's own k, v."""
    b_sz, t_sz, _ = y.shape
    nq, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    pos = np.arange(s0, s0 + t_sz)
    q = (y @ sh.wq).reshape(b_sz, t_sz, nq, d)
    k = (y @ sh.wk).reshape(b_sz, t_sz, nkv, d)
    v = (y @ sh.wv).reshape(b_sz, t_sz, nkv, d)
    q = rope(q, pos, cfg.rope_theta)
    k = rope(k, pos, cfg.rope_theta)
    k = round_storage(k, cfg.storage).transpose(0, 2, 1, 3)    # [B, nkv, T, d]
    v = round_storage(v, cfg.storage).transpose(0, 2, 1, 3)
    if cache_k is None:
        assert s0 == 0
        k_all, v_all = k, v
    else:
        cache_k[:, :, s0:s0 + t_sz] = k
        cache_v[:, :, s0:s0 + t_sz] = v
        k_all, v_all = cache_k, cache_v
    o = causal_gqa_attention(q, k_all, v_all, s0)               # [B, T, nq, d]
    return o.reshape(b_sz, t_sz, nq * d) @ sh.wo


def mlp_partial(y: np.ndarray, sh: ShardLayer) -> np.ndarray:
    """One shard's partial sum of the SwiGLU MLP: (silu(y Wg) * (y Wu)) Wd."""
    return (silu(y @ sh.w_gate) * (y @ sh.w_up)) @ sh.w_down


# ---------------------------------------------------------------------------
# module m = 1..2N and its "AllReduce"
# ---------------------------------------------------------------------------
def module_partials(m: int, u: np.ndarray, layers: Sequence[Layer], cfg: OracleConfig,
                    state: Optional[State], s0: int) -> List[np.ndarray]:
    """Partial sums x*_m of every computed shard for module m on input u [B, T, H]."""
    layer = layers[(m - 1) // 2]
    if m % 2 == 1:
        y = rmsnorm(u, layer.attn_norm, cfg.rms_eps)
        parts = []
        for r, sh in enumerate(layer.shards):
            ck = state.k[(m - 1) // 2][r] if state is not None else None
            cv = state.v[(m - 1) // 2][r] if state is not None else None
            parts.append(attention_partial(y, sh, cfg, s0, ck, cv))
        return parts
    y = rmsnorm(u, layer.mlp_norm, cfg.rms_eps)
    return [mlp_partial(y, sh) for sh in layer.shards]


def all_reduce(m: int, parts: Sequence[np.ndarray], peers: Optional[np.ndarray],
               cfg: OracleConfig) -> np.ndarray:
    """Sum over ranks: computed shards' partials plus, for the ranks that are not
    computed, the synthetic partials peers[m mod pool, j] (rows = (b, t) of this call)."""
    total = np.zeros_like(parts[0])
    for p in parts:
        total = total + p
    if peers is not None:
        b_sz, t_sz, h = total.shape
        pool = peers[m % peers.shape[0]]                 # [n_peers, rows, H]
        for j in range(pool.shape[0]):
            total = total + pool[j, :b_sz * t_sz].reshape(b_sz, t_sz, h)
    return total


def _lags(n_modules: int, wiring) -> List[int]:
    """Input index of module m is m - lag[m]: 2 = ladder (Eq. 2), 1 = standard (Eq. 1).
    `wiring` is "ladder", "standard", "parallel" or a sequence of per-module lags (hybrid).
    "parallel" is the parallel attention / MLP block that section "Faster Inference with Ladder Residual"
    compares with: both modules of a layer read the layer's input and both outputs are added to it, i.e. the
    attention module reads x_{m-1} and the MLP module x_{m-2}."""
    if wiring == "ladder":
        return [2] * n_modules
    if wiring == "standard":
        return [1] * n_modules
    if wiring == "parallel":
        return [1 if m % 2 == 1 else 2 for m in range(1, n_modules + 1)]
    lag = list(wiring)
    assert len(lag) == n_modules and all(v in (1, 2) for v in lag)
    return lag


def forward_eq2(emb: np.ndarray, layers: Sequence[Layer], cfg: OracleConfig,
                state: Optional[State] = None, peers: Optional[np.ndarray] = None,
                wiring="ladder", trace: Optional[dict] = None) -> np.ndarray:
    """Index form.  x_0 = emb [B, T, H];  for m = 1..2N:
         x*_m = h_m(x_{max(m - lag_m, 0)});  x_m = AllReduce(x*_m) + x_{m-1}.
    Returns x_2N.  With `state`, the T tokens are appended at state.pos."""
    emb = np.asarray(emb, dtype=F64)
    n_mod = 2 * cfg.n_layers
    lag = _lags(n_mod, wiring)
    s0 = state.pos if state is not None else 0
    xs = [emb]
    if trace is not None:
        trace.update(x=xs, u=[None], h=[None])
    for m in range(1, n_mod + 1):
        u = xs[max(m - lag[m - 1], 0)]
        h_m = all_reduce(m, module_partials(m, u, layers, cfg, state, s0), peers, cfg)
        xs.append(xs[m - 1] + h_m)
        if trace is not None:
            trace["u"].append(u)
            trace["h"].append(h_m)
    if state is not None:
        state.pos = s0 + emb.shape[1]
    return xs[n_mod]


def forward_alg1(emb: np.ndarray, layers: Sequence[Layer], cfg: OracleConfig,
                 state: Optional[State] = None, peers: Optional[np.ndarray] = None) -> np.ndarray:
    """Variable-passing form (the shape of Algorithm 1; ladder wiring only).  Where `forward_eq2` keeps the
    whole history x_0 .. x_m and indexes it, this form carries what a layer hands to the next one: the stream as
    far as it has been completed, and the module outputs that have been computed but not yet added to it (at
    most two: the paper's attention and MLP outputs in flight).  A module's output is added only when the module
    after next needs the stream, which is where the asynchronous reduction of Algorithm 1 has to have finished.
    Before the first module nothing is outstanding (zero outputs), and after the last one the two outstanding
    outputs are added, oldest first."""
    stream = np.asarray(emb, dtype=F64).copy()     # x_{m-2} when module m starts (x_0 for modules 1 and 2)
    outstanding: List[np.ndarray] = []             # outputs of modules m-2 and m-1, oldest first
    s0 = state.pos if state is not None else 0
    for m in range(1, 2 * cfg.n_layers + 1):
        if len(outstanding) == 2:                  # module m reads x_{m-2} = x_{m-3} + h_{m-2}
            stream = stream + outstanding.pop(0)
        outstanding.append(all_reduce(m, module_partials(m, stream, layers, cfg, state, s0), peers, cfg))
    if state is not None:
        state.pos = s0 + stream.shape[1]
    for h in outstanding:
        stream = stream + h
    return stream


def stage_alg1(residual: np.ndarray, attn_out: Optional[np.ndarray], mlp_out: Optional[np.ndarray],
               layers: Sequence[Layer], cfg: OracleConfig, state: Optional[State] = None,
               peers: Optional[np.ndarray] = None, module_offset: int = 0):
    """One pipeline stage (section "Compatibility with other Parallelism Techniques"): the modules of `layers`
    (cfg.n_layers layers, with their own caches in `state`) in the variable-passing form of `forward_alg1`, except
    that the run neither starts from nothing outstanding nor ends by adding what is: it starts from what the stage
    before hands over and returns what the next stage needs -- three tensors [B, T, H]:

        residual   the stream without the outputs of the last two modules,
        attn_out   the reduced output of the last attention module,
        mlp_out    the reduced output of the last MLP module          (ladder wiring only).

    The first stage gets residual = embeddings and no outputs (None = zeros, which add nothing); the model's
    output x_2N is the sum of the three tensors the last stage returns.  `module_offset` = number of modules in
    the stages before this one; it only selects which synthetic peer partial sums a module's reduction adds."""
    stream = np.asarray(residual, dtype=F64).copy()
    zero = np.zeros_like(stream)
    outstanding = [zero if attn_out is None else np.asarray(attn_out, dtype=F64),     # oldest first: the outputs of
                   zero if mlp_out is None else np.asarray(mlp_out, dtype=F64)]       # the two modules before module 1
    s0 = state.pos if state is not None else 0
    for m in range(1, 2 * cfg.n_layers + 1):
        stream = stream + outstanding.pop(0)       # module m reads the stream up to the output of module m-2
        outstanding.append(all_reduce(module_offset + m, module_partials(m, stream, layers, cfg, state, s0), peers, cfg))
    if state is not None:
        state.pos = s0 + stream.shape[1]
    return stream, outstanding[0], outstanding[1]


# ---------------------------------------------------------------------------
# helpers for tests: build the unsharded model that a set of shards came from
# ---------------------------------------------------------------------------
def merge_shards(layers: Sequence[Layer], cfg: OracleConfig):
    """Concatenate R shards into the single-rank model they partition: first matmuls
    along the output dimension, second matmuls along the input dimension."""
    r = len(layers[0].shards)
    full_cfg = OracleConfig(cfg.n_layers, cfg.hidden, cfg.n_q_heads * r, cfg.n_kv_heads * r, cfg.head_dim,
                            cfg.inter * r, cfg.rms_eps, cfg.rope_theta, cfg.storage, cfg.peer_pool)
    merged = []
    for ly in layers:
        cat_c = lambda name: np.concatenate([getattr(s, name) for s in ly.shards], axis=1)
        cat_r = lambda name: np.concatenate([getattr(s, name) for s in ly.shards], axis=0)
        merged.append(Layer(ly.attn_norm, ly.mlp_norm,
                            [ShardLayer(cat_c("wq"), cat_c("wk"), cat_c("wv"), cat_r("wo"),
                                        cat_c("w_gate"), cat_c("w_up"), cat_r("w_down"))]))
    return merged, full_cfg
