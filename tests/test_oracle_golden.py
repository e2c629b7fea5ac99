"""The oracle still reproduces its stored samples on the seeded tiny workload (drift alarm)."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden"))
import make_tiny_golden as mk  # noqa: E402


def test_tiny_samples_unchanged():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_oracle_samples.txt")
    stored = [ln.split() for ln in open(path) if not ln.startswith("#")]
    rows = mk.run_tiny()
    assert len(rows) == len(stored) == 11
    for (phase, idx, vals), rec in zip(rows, stored):
        assert rec[0] == phase and int(rec[1]) == idx
        assert np.allclose(vals, [float(v) for v in rec[2:]], rtol=0, atol=1e-9)
