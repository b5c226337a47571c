"""The sweep entry point that allocates nothing (static scratch buffer inside the library) against
the entry point that takes a workspace: same kernels, so every output must agree bit for bit.
Two calls in a row, the second on a smaller input, so that whatever the first call left in the
buffer is still there when the second one runs."""
import numpy as np
import pytest

from paper_2001_08743_amd import binding, workloads

pytestmark = pytest.mark.gpu


def _outputs(torch, T, Ksum, n_k, d, ld, n_iter, dev):
    return dict(centroids=torch.full((T, Ksum, d), -7.0, dtype=torch.float64, device=dev),
                counts=torch.full((T, Ksum), -7, dtype=torch.int32, device=dev),
                inertia=torch.full((T, n_k), -7.0, dtype=torch.float64, device=dev),
                status=torch.full((T, n_k), -7, dtype=torch.int32, device=dev),
                labels=torch.full((n_k, ld), 201, dtype=torch.uint8, device=dev),
                trace=torch.full((T, n_k, n_iter + 1), -7.0, dtype=torch.float64, device=dev))


def _compare(wl, flags=0):
    import torch
    dw = binding.DeviceWorkload(wl)
    ref = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                    want_trace=True, flags=flags)
    out = _outputs(torch, wl.T, int(sum(wl.ks)), len(wl.ks), wl.d, dw.ld, wl.n_iter, dw.X.device)
    binding.cham_kmeans_sweep_static(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, out, flags=flags)
    torch.cuda.synchronize()
    for key in ("status", "counts", "centroids", "inertia", "trace"):
        np.testing.assert_array_equal(out[key].cpu().numpy(), ref[key].cpu().numpy(), err_msg=key)
    n = wl.n_total
    np.testing.assert_array_equal(out["labels"].cpu().numpy()[:, :n], ref["labels"].cpu().numpy()[:, :n])


def test_static_scratch_sweep_equals_the_workspace_sweep_on_two_calls_in_a_row():
    binding.cham_static_init()
    big = workloads.make_config(3, 0, scale=0.25)        # 16 tasks x 1024 rows, matrix-core resident kernel
    small = workloads.make_config(1, 1)                  # 256 rows: everything the first call wrote is still there
    _compare(big)
    _compare(small)
    _compare(small, flags=binding.F_NO_MFMA)             # the vector kernel on the same buffer
    mid = workloads.make_config(3, 1, scale=0.125)       # 8 tasks x 1024 rows
    _compare(mid, flags=binding.F_STREAMING)             # the streaming kernels (global sums in the buffer)
    _compare(small, flags=binding.F_STREAMING)


def test_static_scratch_sweep_refuses_inputs_beyond_its_buffer():
    import torch
    wl = workloads.make_config(1, 0)
    dw = binding.DeviceWorkload(wl)
    ks = list(range(2, 34))
    ld = 1 << 18                                          # 256 Ki rows: packed rows alone need 16 MiB
    assert binding.cham_sweep_workspace_bytes(ld, 8, [0, ld], ks, 3) > 8 * 1024 * 1024
    X = torch.zeros((8, ld), dtype=torch.uint8, device=dw.X.device)
    out = _outputs(torch, 1, sum(ks), len(ks), 8, ld, 3, X.device)
    with pytest.raises(binding.ChamError, match="-10"):
        binding.cham_kmeans_sweep_static(X, ld, 8, [0, ld], ks, 3, out)
    torch.cuda.synchronize()
    assert int(out["status"].min()) == -7 and int(out["counts"].max()) == -7      # nothing was written
