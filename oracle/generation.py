"""CPU oracle for the pieces around the block stack that turn it into a token generator.
TEST INFRASTRUCTURE ONLY (same rules as ladder_oracle.py: imported by the tests, the smoke check and
the bench's cpu_baseline leg only; imports nothing from the product).

The paper's inference engine is a prefill followed by token-by-token decoding (section "Inference
Implementation" / "Setup": a gpt-fast style loop on Llama-3 shaped models).  Around the stack of
Ladder-Residual blocks that loop needs, in the Llama-3 architecture:

  * the token embedding: x_0[b, t, :] = table[token[b, t], :]                              (`embed`)
  * the final RMSNorm and the output projection: logits = rmsnorm(x_2N, gain) . W_lm          (`lm_head`)
  * greedy sampling: next token = the index of the largest logit, the lowest index on a tie  (`greedy`)
  * the loop itself: prefill the prompt, then feed every sampled token back                  (`generate`)

Under tensor parallelism the output projection is split along the vocabulary (its output dimension,
the rule of section "Tensor Parallelism Background" for a first matmul): a rank holds V / R columns
and produces V / R logits; nothing else changes, so one function serves both the whole vocabulary
and a rank's slice.  Float64 throughout; the embedding table, the gain and W_lm arrive already rounded
to the storage type.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from . import ladder_oracle as lo

F64 = np.float64


def embed(tokens: np.ndarray, table: np.ndarray) -> np.ndarray:
    """tokens: integer [B, T]; table: [V, H]  ->  [B, T, H]."""
    tokens = np.asarray(tokens)
    if tokens.min() < 0 or tokens.max() >= table.shape[0]:
        raise ValueError("token id outside the table")
    out = np.empty(tokens.shape + (table.shape[1],), dtype=F64)
    for b in range(tokens.shape[0]):
        for t in range(tokens.shape[1]):
            out[b, t] = table[int(tokens[b, t])]
    return out


def lm_head(x: np.ndarray, gain: np.ndarray, w_lm: np.ndarray, eps: float) -> np.ndarray:
    """x: [..., H] residual stream after the last block; gain: [H]; w_lm: [H, V]  ->  logits [..., V]."""
    return lo.rmsnorm(np.asarray(x, dtype=F64), gain, eps) @ w_lm


def greedy(logits: np.ndarray) -> np.ndarray:
    """Index of the largest logit along the last axis; the lowest index among equal maxima."""
    flat = logits.reshape(-1, logits.shape[-1])
    out = np.empty(flat.shape[0], dtype=np.int64)
    for r in range(flat.shape[0]):
        best, at = flat[r, 0], 0
        for v in range(1, flat.shape[1]):
            if flat[r, v] > best:
                best, at = flat[r, v], v
        out[r] = at
    return out.reshape(logits.shape[:-1])


def generate(prompt: np.ndarray, n_new: int, table: np.ndarray, gain: np.ndarray, w_lm: np.ndarray,
             layers: Sequence[lo.Layer], cfg: lo.OracleConfig, state: lo.State,
             peers_prefill: Optional[np.ndarray] = None, peers_decode: Optional[np.ndarray] = None,
             wiring="ladder"):
    """Greedy generation: prefill `prompt` [B, T], then n_new tokens one at a time through the KV cache.
    Returns (tokens [B, n_new], logits of every sampled position [n_new][B, V])."""
    x = lo.forward_eq2(embed(prompt, table), layers, cfg, state, peers_prefill, wiring=wiring)
    logits = lm_head(x[:, -1], gain, w_lm, cfg.rms_eps)
    toks: List[np.ndarray] = []
    all_logits: List[np.ndarray] = []
    for i in range(n_new):
        nxt = greedy(logits)
        toks.append(nxt)
        all_logits.append(logits)
        if i + 1 == n_new:
            break
        x = lo.forward_eq2(embed(nxt[:, None], table), layers, cfg, state, peers_decode, wiring=wiring)
        logits = lm_head(x[:, 0], gain, w_lm, cfg.rms_eps)
    return np.stack(toks, axis=1), all_logits
