"""Shared glue for the tests: seeded inputs -> oracle structures (CPU side)."""
from __future__ import annotations

import numpy as np

from oracle import from_torch
from oracle import ladder_oracle as lo
from paper_2501_06589_amd import inputs


def oracle_model(w: inputs.Workload, n_layers=None, device="cpu", tensors=None):
    """Oracle layers (lazy) + config for workload `w`.  `tensors`, if given, is
    tensors[layer][shard] -> dict of torch tensors already generated elsewhere."""
    n_layers = n_layers or w.n_layers
    cfg = from_torch.config_from_workload(w)
    cfg.n_layers = n_layers

    def make(i):
        if tensors is not None:
            return from_torch.layer_from_tensors(tensors[i])
        return from_torch.layer_from_tensors([inputs.layer_weights(w, i, r, device) for r in range(w.n_real_shards)])

    return from_torch.LazyLayers(n_layers, make), cfg


def rel_err(got, want) -> float:
    """max |got - want| / RMS(want)"""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(got - want)) / np.sqrt(np.mean(want * want)))
