"""GPU parity of the chained decode step (decode_fused = 3): the whole launch list of a step in one launch of
persistent workgroups, the jobs meeting at flags instead of launch boundaries.  The arithmetic and its order are
those of the launch list, so the results are bit-identical to the launch-per-job schedules; against the oracle the
bar is the bf16-storage one (max |gpu - oracle| / RMS(oracle) < 2e-2 on every call's final x_2N).
"""
import numpy as np
import pytest
import torch

from paper_2501_06589_amd import inputs, ladder

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
R8_SMALL = inputs.WORKLOADS["70b_r8_decode"].with_(name="r8_small", n_layers=3, hidden=512, inter=448, batch=4,
                                                   decode_steps=6)


@pytest.fixture(scope="module")
def harness():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("wiring,nstd", [(ladder.LADDER_WIRING_LADDER, 0), (ladder.LADDER_WIRING_STANDARD, 0),
                                         (ladder.LADDER_WIRING_LADDER, 2), (ladder.LADDER_WIRING_PARALLEL, 0)])
def test_chained_step_matches_oracle_and_the_launch_list(harness, wiring, nstd):
    """Every wiring (Algorithm 1, Eq. 1, the hybrid stack, the parallel block), synthetic peers, preloaded cache,
    decode crossing a 32-position boundary: against the oracle, and bit for bit against the same launch list run
    as separate launches."""
    kw = dict(kv_preload=125 if nstd else 700, wiring=wiring, n_standard_layers=nstd)
    res = harness.run_case(R8_SMALL, decode_fused=3, **kw)
    assert len(res.errs) == 6 and max(res.errs) < TOL_BF16, res.errs
    ref = harness.run_case(R8_SMALL, gpu_only=True, decode_fused=1, **kw)
    for x, y in zip(res.gpu, ref.gpu):
        assert np.array_equal(x, y)
