"""Seeded synthetic inputs for the Ladder-Residual shard forward.

This module only *draws numbers* and names workload shapes.  It holds none of
the method's arithmetic (no norm, no rotation, no attention, no reduction) and
is the single piece of code that both the CPU oracle's tests and the HIP path's
tests/bench may use, so that both sides see bit-identical inputs.

Generator.  Every element of every tensor is a pure function of
``(seed, tensor_id, flat_index)``: two 32-bit avalanche hashes give two
uniforms, Box-Muller (float64) turns them into one standard normal, which is
scaled, shifted and finally rounded to the storage dtype (fp32 or bf16, RNE via
torch's cast).  It is written with torch integer/elementwise ops only, so the
same code runs on the CPU (tests) and on the GPU (multi-GB weight sets that
must be created in seconds).  All integer arithmetic stays below 2**63, so no
step relies on wrap-around.  A tensor that must be identical on both sides is
generated once and copied, never generated twice on different devices
(float64 log/cos may differ by an ulp between libraries).

Recipe: projection weights N(0, 0.02^2);
norm gains 1 + 0.02*N(0,1) (so that a forgotten gain multiply is visible);
input embeddings N(0,1); synthetic peer partials N(0, 0.02^2); synthetic
KV-cache entries N(0,1).  Seeds: 0 weights, 1 prefill embeddings, 2+step
decode embeddings, 100 peers, 200 KV cache.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import torch

_M32 = 0xFFFFFFFF

# tensor kinds (part of tensor_id)
ATTN_NORM, WQ, WK, WV, WO, MLP_NORM, W_GATE, W_UP, W_DOWN = range(9)
KV_K, KV_V = 10, 11

SEED_WEIGHTS = 0
SEED_PREFILL = 1
SEED_DECODE0 = 2          # + step
SEED_PEERS = 100
SEED_KV = 200


def _mul32(x: torch.Tensor, c: int) -> torch.Tensor:
    """(x * c) mod 2**32 for int64 x in [0, 2**32) without exceeding 2**63."""
    lo = x * (c & 0xFFFF)
    hi = (x * (c >> 16)) & 0xFFFF
    return (lo + (hi << 16)) & _M32


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche hash (xorshift-multiply, two rounds) on int64 lanes."""
    x = x ^ (x >> 16)
    x = _mul32(x, 0x7FEB352D)
    x = x ^ (x >> 15)
    x = _mul32(x, 0x846CA68B)
    x = x ^ (x >> 16)
    return x


def _mix32_scalar(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & _M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & _M32
    x ^= x >> 16
    return x


def _stream_keys(seed: int, tensor_id: int):
    a = _mix32_scalar(seed * 0x9E3779B1 + 0x1234567)
    b = _mix32_scalar(a ^ (tensor_id & _M32))
    c = _mix32_scalar(b + (tensor_id >> 32) + 0x632BE5AB)
    k1 = _mix32_scalar(c ^ 0xA5A5A5A5)
    k2 = _mix32_scalar(c ^ 0x3C3C3C3C)
    return k1, k2


def normal(seed: int, tensor_id: int, shape, *, std: float = 1.0, mean: float = 0.0,
           dtype: torch.dtype = torch.float32, device="cpu",
           chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of ``shape`` with element i = mean + std * z(seed, tensor_id, i)."""
    shape = tuple(int(s) for s in shape)
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(n, dtype=dtype, device=device)
    k1, k2 = _stream_keys(seed, tensor_id)
    for start in range(0, n, chunk):
        stop = min(n, start + chunk)
        idx = torch.arange(start, stop, dtype=torch.int64, device=device)
        lo = idx & _M32
        hi = idx >> 32
        h1 = _mix32(_mix32(lo ^ k1) ^ _mul32(hi + 1, 0x27D4EB2F))
        h2 = _mix32(_mix32(lo ^ k2) ^ _mul32(hi + 1, 0x165667B1))
        u1 = (h1.to(torch.float64) + 0.5) * (1.0 / 4294967296.0)
        u2 = (h2.to(torch.float64) + 0.5) * (1.0 / 4294967296.0)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[start:stop] = (z * std + mean).to(dtype)
    return out.view(shape)


# --------------------------------------------------------------------------
# workload shapes (per-shard, i.e. local sizes)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "fp32" | "bf16"
    n_layers: int
    hidden: int
    n_q_heads: int        # local (per shard)
    n_kv_heads: int       # local
    head_dim: int
    inter: int            # local SwiGLU intermediate
    tp_degree: int        # R
    n_real_shards: int    # shards computed for real (R or 1); the rest are synthetic peers
    batch: int
    prefill: int          # prompt tokens per sequence (0: synthetic cache instead)
    kv_preload: int       # tokens of synthetic KV cache loaded before decode
    decode_steps: int
    rope_theta: float
    rms_eps: float = 1e-5
    peer_pool: int = 2

    @property
    def n_peers(self) -> int:
        return self.tp_degree - self.n_real_shards

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    @property
    def max_seq(self) -> int:
        return self.prefill + self.kv_preload + self.decode_steps

    def params_per_layer(self) -> int:
        """Projection-matrix parameters of ONE shard of one layer."""
        h, d = self.hidden, self.head_dim
        return (h * (self.n_q_heads + 2 * self.n_kv_heads) * d
                + self.n_q_heads * d * h + 3 * h * self.inter)

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # tiny ladder model, fp32, both TP shards computed for real
    "tiny": Workload("tiny", "fp32", 2, 256, 2, 1, 64, 344, 2, 2, 1, 32, 0, 8, 1e4, peer_pool=1),
    # 1.2B-class, whole model on one GPU
    "1.2b": Workload("1.2b", "bf16", 24, 2048, 16, 8, 128, 5632, 1, 1, 4, 1024, 0, 128, 1e4, peer_pool=1),
    # Llama-3.1-8B-shaped
    "8b": Workload("8b", "bf16", 32, 4096, 32, 8, 128, 14336, 1, 1, 4, 2048, 0, 128, 5e5, peer_pool=1),
    # 70B-shaped single TP rank at R=8: decode headline
    "70b_r8_decode": Workload("70b_r8_decode", "bf16", 80, 8192, 8, 1, 128, 3584, 8, 1, 4, 0, 1024,
                              256, 5e5, peer_pool=2),
    # 70B-shaped single TP rank at R=4: prefill-heavy
    "70b_r4_prefill": Workload("70b_r4_prefill", "bf16", 80, 8192, 16, 2, 128, 7168, 4, 1, 16, 2048, 0,
                               128, 5e5, peer_pool=2),
}


def tensor_id(layer: int, shard: int, kind: int) -> int:
    return (layer * 64 + shard) * 16 + kind


def layer_weights(w: Workload, layer: int, shard: int, device="cpu",
                  seed: int = SEED_WEIGHTS) -> Dict[str, torch.Tensor]:
    """Weights of one shard of one layer, in the caller-side layout of the C-ABI:
    row-major ``[in_features, out_features]`` (row-vector convention y = x W)."""
    dt = w.torch_dtype
    h, d, i = w.hidden, w.head_dim, w.inter
    nq, nkv = w.n_q_heads, w.n_kv_heads

    def mat(kind, rows, cols):
        return normal(seed, tensor_id(layer, shard, kind), (rows, cols), std=0.02, dtype=dt, device=device)

    def gain(kind):
        # gains are replicated over shards: shard index 0 in the id
        return normal(seed, tensor_id(layer, 0, kind), (h,), std=0.02, mean=1.0, dtype=dt, device=device)

    return {
        "attn_norm": gain(ATTN_NORM),
        "wq": mat(WQ, h, nq * d), "wk": mat(WK, h, nkv * d), "wv": mat(WV, h, nkv * d),
        "wo": mat(WO, nq * d, h),
        "mlp_norm": gain(MLP_NORM),
        "w_gate": mat(W_GATE, h, i), "w_up": mat(W_UP, h, i), "w_down": mat(W_DOWN, i, h),
    }


def embeddings(w: Workload, batch: int, tokens: int, seed: int, device="cpu") -> torch.Tensor:
    """Input embeddings [batch, tokens, hidden] ~ N(0,1) in the storage dtype."""
    return normal(seed, 0, (batch, tokens, w.hidden), dtype=w.torch_dtype, device=device)


def peer_partials(w: Workload, rows: int, device="cpu", seed: int = SEED_PEERS) -> Optional[torch.Tensor]:
    """Synthetic partial sums of the ranks that are not computed:
    [peer_pool, R - n_real, rows, hidden] ~ N(0, 0.02^2)."""
    if w.n_peers == 0:
        return None
    return normal(seed, 0, (w.peer_pool, w.n_peers, rows, w.hidden), std=0.02,
                  dtype=w.torch_dtype, device=device)


def kv_cache(w: Workload, layer: int, shard: int, batch: int, tokens: int, device="cpu",
             seed: int = SEED_KV) -> List[torch.Tensor]:
    """Synthetic cache content for one layer/shard: K (taken as already rotated) and V,
    each [batch, n_kv_heads, tokens, head_dim] ~ N(0,1)."""
    shp = (batch, w.n_kv_heads, tokens, w.head_dim)
    return [normal(seed, tensor_id(layer, shard, kind), shp, dtype=w.torch_dtype, device=device)
            for kind in (KV_K, KV_V)]


# ---- generation head (token embedding, final norm, output projection) ---------------------------
SEED_HEAD = 300
SEED_PROMPT = 400
HEAD_TABLE, HEAD_GAIN, HEAD_WLM = 1, 2, 3


def head_weights(w: Workload, vocab: int, vocab_local: Optional[int] = None, shard: int = 0, device="cpu",
                 seed: int = SEED_HEAD) -> Dict[str, torch.Tensor]:
    """Token embedding table [vocab, hidden] ~ N(0,1), final norm gain [hidden] ~ 1 + 0.02 N(0,1) and this
    rank's slice of the output projection [hidden, vocab_local] ~ N(0, 0.02^2) (vocabulary-parallel split:
    rank `shard` owns columns shard * vocab_local ...)."""
    dt = w.torch_dtype
    vl = vocab if vocab_local is None else vocab_local
    return {
        "table": normal(seed, HEAD_TABLE, (vocab, w.hidden), dtype=dt, device=device),
        "final_norm": normal(seed, HEAD_GAIN, (w.hidden,), std=0.02, mean=1.0, dtype=dt, device=device),
        "w_lm": normal(seed, tensor_id(0, shard, HEAD_WLM), (w.hidden, vl), std=0.02, dtype=dt, device=device),
    }


def prompt_tokens(batch: int, tokens: int, vocab: int, device="cpu", seed: int = SEED_PROMPT) -> torch.Tensor:
    """Seeded token ids [batch, tokens], int32, uniform over the vocabulary (from the same counter hash)."""
    u = normal(seed, 0, (batch, tokens), dtype=torch.float64, device=device)
    # the normal deviate's CDF is uniform: Phi(u) in (0, 1)
    p = 0.5 * (1.0 + torch.erf(u / 2.0 ** 0.5))
    return torch.clamp((p * vocab).to(torch.int64), 0, vocab - 1).to(torch.int32)
