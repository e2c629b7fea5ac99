"""Glue for tests and the bench's cpu_baseline leg: torch tensors (as produced by the
seeded input generator) -> the oracle's float64 numpy structures.  No arithmetic."""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

from .ladder_oracle import Layer, OracleConfig, ShardLayer, State


def to_f64(t) -> np.ndarray:
    return t.detach().to("cpu").double().numpy()


def layer_from_tensors(shards: Sequence[Dict[str, "object"]]) -> Layer:
    """shards[r] is the dict {attn_norm, wq, wk, wv, wo, mlp_norm, w_gate, w_up, w_down}
    of rank r; the gains are taken from rank 0 (they are replicated)."""
    sl = [ShardLayer(*(to_f64(s[k]) for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")))
          for s in shards]
    return Layer(to_f64(shards[0]["attn_norm"]), to_f64(shards[0]["mlp_norm"]), sl)


class LazyLayers:
    """Sequence of layers built on demand (one kept alive), so that a multi-GB model
    never has to exist in float64 all at once."""

    def __init__(self, n_layers: int, make_layer):
        self._n, self._make, self._cached = n_layers, make_layer, (None, None)

    def __len__(self):
        return self._n

    def __getitem__(self, i: int) -> Layer:
        if self._cached[0] != i:
            self._cached = (i, self._make(i))
        return self._cached[1]


def config_from_workload(w, storage: str = None) -> OracleConfig:
    return OracleConfig(w.n_layers, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.inter,
                        w.rms_eps, w.rope_theta, storage or w.dtype, w.peer_pool)


def load_kv(state: State, layer: int, shard: int, k, v) -> None:
    """Copy synthetic cache content [B, nkv, S, d] into the oracle state."""
    s = k.shape[2]
    state.k[layer][shard][:, :, :s] = to_f64(k)
    state.v[layer][shard][:, :, :s] = to_f64(v)
