"""Randomised parity: the whole path on workloads of random shape against the oracle, through every
sweep kernel family (the flags are drawn with the workload)."""
import numpy as np
import pytest

from paper_2001_08743_amd import binding, workloads
from parity_util import check_pipeline, check_sweep, knee_margin, run_both

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(6))
def test_random_workloads_match_the_oracle(block):
    seen_paths = set()
    for seed in range(40 * block, 40 * block + 40):
        wl = workloads.random_workload(seed)
        wide = wl.rows.dtype == np.uint16
        rng = np.random.default_rng(seed)
        if wide:
            flags = int(rng.choice([0, 0, binding.F_NO_MFMA]))
        else:
            flags = int(rng.choice([0, 0, 0, binding.F_NO_MFMA, binding.F_STREAMING, binding.F_RESIDENT]))
        ld = (wl.n_total + 63) // 64 * 64
        promise = binding.F_VALUES_BELOW_2048 if wide and int(wl.cards.max()) <= 2048 else 0
        seen_paths.add((wide, binding.cham_sweep_path(ld, wl.d, wl.task_off, wl.ks, flags | promise,
                                                      _sfx="_u16" if wide else "")))
        dw, g, c = run_both(wl, flags=flags)
        try:
            check_sweep(wl, g["sweep"], c, dw.ld)
            # the chosen k is compared where no threshold test of the loss curve sits at equality
            if all(knee_margin(c["inertia"][t], c["status"][t], wl.threshold) > 1e-9 or c["inertia"][t].max() == 0
                   for t in range(wl.T)):
                check_pipeline(wl, g, c)
        except AssertionError as e:
            raise AssertionError(f"workloads.random_workload({seed}), flags {flags}: {e}") from e
    # every kernel family took part: byte knobs on all three, two-byte knobs on the matrix cores and the vector ALU
    assert {(False, 0), (False, 1), (False, 2), (True, 2)} <= seen_paths
