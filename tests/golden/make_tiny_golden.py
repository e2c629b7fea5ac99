"""Writes tests/golden/tiny_oracle_samples.txt: sampled outputs of the CPU oracle on the
seeded "tiny" workload (fp32 storage, 2 ladder layers, R = 2 real shards, batch 1,
prefill 32 tokens, 8 decode steps).  Calls only oracle/ and the seeded input generator.
The paper prints no numeric example; this fixture is a drift alarm for the oracle, it
is not evidence that the oracle is right (the pins are).

Run:  python tests/golden/make_tiny_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import from_torch                      # noqa: E402
from oracle import ladder_oracle as lo             # noqa: E402
from paper_2501_06589_amd import inputs            # noqa: E402

SAMPLE_COLS = [0, 1, 17, 100, 255]


def run_tiny():
    w = inputs.WORKLOADS["tiny"]
    cfg = from_torch.config_from_workload(w)
    layers = [from_torch.layer_from_tensors([inputs.layer_weights(w, i, r) for r in range(w.n_real_shards)])
              for i in range(w.n_layers)]
    state = lo.State.empty(cfg, w.n_real_shards, w.batch, w.max_seq)
    rows = []
    out = lo.forward_eq2(from_torch.to_f64(inputs.embeddings(w, w.batch, w.prefill, inputs.SEED_PREFILL)),
                         layers, cfg, state)
    for t in (0, 15, 31):
        rows.append(("prefill", t, out[0, t, SAMPLE_COLS]))
    for step in range(w.decode_steps):
        e = from_torch.to_f64(inputs.embeddings(w, w.batch, 1, inputs.SEED_DECODE0 + step))
        out = lo.forward_eq2(e, layers, cfg, state)
        rows.append(("decode", step, out[0, 0, SAMPLE_COLS]))
    return rows


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle_samples.txt")
    with open(path, "w") as f:
        f.write("# oracle forward_eq2 on workload 'tiny'; columns %s of x_2N; written by make_tiny_golden.py\n" % SAMPLE_COLS)
        for phase, idx, vals in run_tiny():
            f.write("%s %d %s\n" % (phase, idx, " ".join("%.12e" % v for v in vals)))
    print("wrote", path)
