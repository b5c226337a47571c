"""The full-model sweep at the size and in the launch the benchmark times (256 tasks x 4096
configurations x 24 knobs, k = 1..64 in one call), every task against the CPU oracle: sweep outputs,
chosen k, picks, synthesized configurations (Algorithm 1 per task).  The oracle needs about a minute on
the GPU machine's host cores; the file name puts the test near the end of the run."""
import numpy as np
import pytest

import oracle
from paper_2001_08743_amd import binding, workloads
from parity_util import check_pipeline, check_sweep, oracle_visited

pytestmark = pytest.mark.gpu


def test_cfg5_every_task_against_the_oracle():
    import torch
    wl = workloads.make_config(5, 0)
    dw = binding.DeviceWorkload(wl)
    dw.build_visited()
    res = dw.run()                                  # the bench's launch: no label or trace output
    torch.cuda.synchronize()
    vis = oracle_visited(wl)
    np.testing.assert_array_equal(dw.visited_host, vis)
    chunk = 32                                      # tasks per oracle call: progress output, bounded memory
    for t0 in range(0, wl.T, chunk):
        tasks = list(range(t0, min(t0 + chunk, wl.T)))
        sub = wl.subset(tasks)
        ref = oracle.pipeline(sub, vis)
        sl = slice(tasks[0], tasks[-1] + 1)
        r0, r1 = int(wl.task_off[tasks[0]]), int(wl.task_off[tasks[-1] + 1])
        got = dict(sweep={k: res["sweep"][k][sl] for k in ("centroids", "counts", "inertia", "status")},
                   chosen=res["chosen"][sl],
                   snap=dict(labels_sel=res["snap"]["labels_sel"][r0:r1], pick_row=res["snap"]["pick_row"][sl],
                             pick_cfg=res["snap"]["pick_cfg"][sl]),
                   synth={k: res["synth"][k][sl] for k in ("out_cfg", "out_flag", "out_count")})
        check_sweep(sub, got["sweep"], ref, dw.ld, check_labels=False)
        check_pipeline(sub, got, ref)
        print(f"cfg5 tasks {tasks[0]}..{tasks[-1]} match the oracle", flush=True)
    # the sweep stopped every unit at its fixed point or at the last pass
    passes = binding.cham_sweep_passes(res["sweep"]["workspace"], dw.ld, dw.d, wl.task_off, wl.ks).cpu().numpy()
    assert passes.min() >= 1 and passes.max() <= wl.n_iter + 1
