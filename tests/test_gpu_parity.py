"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from paper_2001_08743_amd import binding, workloads
from parity_util import check_pipeline, check_sweep, knee_margin, oracle_visited, run_both

pytestmark = pytest.mark.gpu


def _full(wl, threshold=None, flags=0, want_trace=False):
    dw, g, c = run_both(wl, threshold=threshold, flags=flags, want_trace=want_trace)
    check_sweep(wl, g["sweep"], c, dw.ld)
    thr = wl.threshold if threshold is None else threshold
    for t in range(wl.T):
        # the knee decision must not sit on a rounding-sensitive equality for the seeds used here
        assert knee_margin(c["inertia"][t], c["status"][t], thr) > 1e-9 or c["inertia"][t].max() == 0
    check_pipeline(wl, g, c)
    return dw, g, c


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg1_tiny(seed):
    _full(workloads.make_config(1, seed), want_trace=True)


@pytest.mark.parametrize("thr", [1.0, 1.05, 1.5])
def test_cfg1_other_thresholds(thr):
    _full(workloads.make_config(1, 0), threshold=thr)


def test_cfg1_force_exact():
    _full(workloads.make_config(1, 0), flags=binding.F_FORCE_EXACT)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg2_conv2d(seed):
    _full(workloads.make_config(2, seed))


@pytest.mark.parametrize("thr", [1.0, 1.05, 1.5])
def test_cfg2_other_thresholds(thr):
    wl = workloads.make_config(2, 0)
    wl.n_iter = 12
    _full(wl, threshold=thr)


@pytest.mark.parametrize("seed", [0, 1])
def test_cfg3_batched_quarter(seed):
    _full(workloads.make_config(3, seed, scale=0.25))


def test_cfg5_two_tasks():
    wl = workloads.make_config(5, 0, scale=2 / 256)
    wl.n_iter = 20
    _full(wl)


@pytest.mark.parametrize("d", [1, 3, 4, 13, 17, 28, 32])
def test_knob_counts(d):
    wl = workloads.random_task(900 + d, n=700, d=d, n_blobs=5, ks=(1, 2, 5, 9), n_iter=8, n_visited=64,
                               invalid_frac=0.1, n_tasks=2, ragged=True, card_hi=30)
    _full(wl, threshold=1.05)


def test_ragged_unaligned_tasks_and_tiny_tasks():
    rng = np.random.default_rng(5)
    sizes = [1, 2, 3, 5, 130, 257, 1023, 7]
    cards = [rng.integers(2, 9, size=6).astype(np.uint16) for _ in sizes]
    wl = workloads._assemble("ragged", rng, sizes, cards, [3] * len(sizes), 1.0, 0.1, (1, 2, 3, 4), 6, 32)
    _full(wl, threshold=1.2)


def test_k_up_to_256():
    wl = workloads.random_task(31, n=3000, d=8, n_blobs=40, card_hi=32, sigma=1.5, ks=(64, 200, 256), n_iter=5,
                               n_visited=128, invalid_frac=0.05)
    _full(wl, threshold=1.01)


def test_multi_tile_task():
    # more rows than one workgroup tile (4096): the tile loop and cross-tile label storage
    wl = workloads.random_task(32, n=9001, d=12, n_blobs=12, card_hi=20, sigma=1.5, ks=(3, 17), n_iter=6,
                               n_visited=64)
    _full(wl, threshold=1.01)


def test_duplicate_heavy_rows_exact_ties():
    # few distinct rows, many exact distance ties: every decision must follow the lowest-index rule
    rng = np.random.default_rng(9)
    base = rng.integers(0, 4, size=(9, 5)).astype(np.uint8)
    rows = base[rng.integers(0, 9, size=600)]
    wl = workloads.random_task(1, n=8, d=5)
    wl.rows, wl.task_off = np.ascontiguousarray(rows), np.array([0, 600])
    wl.valid = np.ones(600, np.uint8)
    wl.cards = np.full((1, 5), 4, np.uint16)
    wl.ks, wl.n_iter = [1, 2, 4, 8, 12], 7
    dw, g, c = _full(wl, threshold=1.3)
    assert c["status"][0, -1] == 1          # fewer than 12 distinct rows


def test_caller_supplied_start_single_step():
    """Teacher-forced step: oracle centroids in, one Lloyd step, compare labels, counts, centroids."""
    import torch
    wl = workloads.make_config(2, 0)
    wl.ks, wl.n_iter = [5, 16, 40], 3
    sw0 = oracle.sweep(wl.rows, wl.task_off, wl.ks, 3)
    init = sw0["centroids"]
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, 1, init=init, want_labels=True)
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, 1,
                                    init_centroids=torch.from_numpy(init).to(dw.device), want_labels=True)
    torch.cuda.synchronize()
    check_sweep(wl, out, ref, dw.ld)


def test_run_twice_bit_identical():
    import torch
    wl = workloads.make_config(3, 0, scale=0.125)
    dw = binding.DeviceWorkload(wl)
    a = dw.run(want_labels=True)
    b = dw.run(want_labels=True)
    torch.cuda.synchronize()
    for key in ("centroids", "counts", "inertia", "status", "labels"):
        assert torch.equal(a["sweep"][key], b["sweep"][key]), key
    assert torch.equal(a["synth"]["out_cfg"], b["synth"]["out_cfg"])


def test_hash_rows_matches_host_hash():
    import torch
    rng = np.random.default_rng(3)
    rows = rng.integers(0, 256, size=(1000, 11)).astype(np.uint8)
    salts = rng.integers(0, 2 ** 62, size=1000).astype(np.int64)
    h = binding.cham_hash_rows(torch.from_numpy(rows).cuda(), torch.from_numpy(salts).cuda()).cpu().numpy().view(np.uint64)
    ref = oracle.hash_rows(rows, salts.astype(np.uint64))
    np.testing.assert_array_equal(h, ref)
    assert binding.cham_hash_config(rows[0], int(salts[0])) == int(ref[0])


# ------------------------------------------------------------------ full benchmark sizes

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cfg3_full_size(seed):
    _full(workloads.make_config(3, seed))


def test_cfg4_full_size():
    """One clustering of 1,048,576 rows: the oracle runs the whole sweep (OpenMP over rows)."""
    wl = workloads.make_config(4, 0)
    _full(wl)


def test_cfg5_full_size_sampled_tasks():
    """The launch the bench times (256 tasks x 64 k values in one call); the oracle recomputes a
    sample of whole tasks, which are independent of each other."""
    import torch
    wl = workloads.make_config(5, 0)
    dw = binding.DeviceWorkload(wl)
    dw.build_visited()
    res = dw.run(want_labels=True)
    torch.cuda.synchronize()
    from parity_util import oracle_visited
    vis = oracle_visited(wl)
    np.testing.assert_array_equal(dw.visited_host, vis)
    sample = [0, 101, 255]
    sub = wl.subset(sample)
    sw_cpu = oracle.sweep(sub.rows, sub.task_off, sub.ks, sub.n_iter, want_labels=True)
    ref = oracle.pipeline(sub, vis, sweep_out=sw_cpu)
    sw = res["sweep"]
    for i, t in enumerate(sample):
        r0, r1 = wl.task_off[t], wl.task_off[t + 1]
        s0, s1 = sub.task_off[i], sub.task_off[i + 1]
        np.testing.assert_array_equal(sw["counts"][t].cpu().numpy(), ref["counts"][i])
        np.testing.assert_array_equal(sw["centroids"][t].cpu().numpy(), ref["centroids"][i])
        np.testing.assert_allclose(sw["inertia"][t].cpu().numpy(), ref["inertia"][i], rtol=1e-11, atol=0)
        np.testing.assert_array_equal(sw["labels"][:, r0:r1].cpu().numpy().astype(np.int32), ref["labels"][:, s0:s1])
        assert int(res["chosen"][t]) == int(ref["chosen_idx"][i])
        np.testing.assert_array_equal(res["snap"]["labels_sel"][r0:r1].cpu().numpy().astype(np.int32), ref["labels_sel"][s0:s1])
        np.testing.assert_array_equal(res["snap"]["pick_row"][t].cpu().numpy().astype(np.int64), ref["pick_row"][i])
        np.testing.assert_array_equal(res["synth"]["out_cfg"][t].cpu().numpy(), ref["out_cfg"][i])
        np.testing.assert_array_equal(res["synth"]["out_flag"][t].cpu().numpy(), ref["out_flag"][i])
        assert int(res["synth"]["out_count"][t]) == int(ref["out_count"][i])
    # properties that hold for every task at any size
    counts = sw["counts"].cpu().numpy()
    koff = sw["koff"]
    for ki, k in enumerate(wl.ks):
        assert (counts[:, koff[ki]:koff[ki] + k].sum(axis=1) == 4096).all()
    inertia = sw["inertia"].cpu().numpy()
    assert (inertia >= 0).all()


# ------------------------------------------------------------------ matrix-core path specifics

@pytest.mark.parametrize("d,k", [(13, 32), (14, 33), (15, 32), (16, 33), (29, 64), (30, 64), (31, 64), (24, 1),
                                 (2, 64)])
def test_matrix_core_path_boundaries(d, k):
    """Knob counts around the 16/32 fragment widths (the resident kernel keeps the last slot for the
    bias: 15 and 31 knobs are its limits per width) and centroid counts around the 32-row tile."""
    wl = workloads.random_task(700 + d + k, n=1500, d=d, n_blobs=max(2, k // 2), ks=(k,), n_iter=7,
                               n_visited=32, card_hi=24, sigma=1.3)
    _full(wl, threshold=1.01)


@pytest.mark.parametrize("n", [4095, 4096, 4097])
def test_row_counts_around_the_resident_limit(n):
    wl = workloads.random_task(40 + n, n=n, d=9, n_blobs=7, ks=(3, 40), n_iter=5, n_visited=16)
    _full(wl, threshold=1.01)


def test_every_row_on_an_exact_tie_overflows_the_queue():
    """All rows are equidistant from two caller-supplied centroids: every row is inside the error
    bound, far more than a wave's queue keeps in LDS, and must get the lowest index."""
    import torch
    n, d = 4096, 6
    rows = np.full((n, d), 4, dtype=np.uint8)
    rows[::7, 0] = 5                      # a few rows off the tie so that later passes differ
    wl = workloads.random_task(3, n=8, d=d)
    wl.rows, wl.task_off = rows, np.array([0, n])
    wl.valid = np.ones(n, np.uint8)
    wl.cards = np.full((1, d), 16, np.uint16)
    wl.ks, wl.n_iter = [2, 3], 3
    init = np.zeros((1, 5, d))
    init[0, 0] = 2.0
    init[0, 1] = 6.0                      # k = 2: all rows with value 4 tie exactly
    init[0, 2] = 2.0
    init[0, 3] = 6.0
    init[0, 4] = 6.0                      # k = 3: centroids 1 and 2 coincide as well
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, init=init, want_labels=True, want_trace=True)
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter,
                                    init_centroids=torch.from_numpy(init).to(dw.device), want_labels=True,
                                    want_trace=True)
    torch.cuda.synchronize()
    check_sweep(wl, out, ref, dw.ld)


@pytest.mark.parametrize("seed,d,card_hi,ks", [(801, 3, 3, (2, 5, 9)), (802, 6, 4, (7, 33, 40)), (803, 24, 8, (16, 64))])
def test_many_passes_after_convergence_with_ties(seed, d, card_hi, ks):
    """Few distinct values per knob: many duplicate rows and exact ties, and the sweep runs long
    after the centroids have stopped moving, so most passes only count the scores below each row's
    threshold and re-resolve the tied rows exactly."""
    wl = workloads.random_task(seed, n=4096, d=d, card_hi=card_hi, n_blobs=5, sigma=2.0, ks=ks, n_iter=40,
                               n_tasks=2, ragged=True)
    _sweep_only(wl, 0, want_trace=True)


def test_converged_start_counts_from_the_second_pass():
    """Caller-supplied centroids that are already a fixed point: no pass changes a centroid."""
    import torch
    wl = workloads.random_task(810, n=3000, d=10, n_blobs=6, ks=(6,), n_iter=60, card_hi=12)
    ref0 = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    init = ref0["centroids"].reshape(1, 6, 10).copy()
    wl.n_iter = 12
    _sweep_only(wl, 0, want_trace=True, init=init)


def test_full_model_sweep_matrix_core_equals_vector_path():
    """The whole benchmark workload (256 tasks, every k): the matrix-core kernel, which stops at the
    fixed point, and the vector kernel, which runs every pass, must agree bit for bit on every
    unit, and every unit reports status 0."""
    import torch
    wl = workloads.make_config(5, 0)
    dw = binding.DeviceWorkload(wl)
    a = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True)
    b = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                  flags=binding.F_NO_MFMA)
    torch.cuda.synchronize()
    assert int(a["status"].abs().sum().item()) == 0
    for key in ("centroids", "counts", "status", "labels"):
        assert torch.equal(a[key], b[key]), key
    np.testing.assert_allclose(a["inertia"].cpu().numpy(), b["inertia"].cpu().numpy(), rtol=1e-12, atol=0)


def test_matrix_core_and_vector_paths_agree_on_every_task():
    """The two screens must lead to identical results (both are exact); this covers all tasks of a
    slice of the full-model workload, beyond what the oracle samples."""
    import torch
    wl = workloads.make_config(5, 0, scale=16 / 256)
    dw = binding.DeviceWorkload(wl)
    a = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True)
    b = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                  flags=binding.F_NO_MFMA)
    torch.cuda.synchronize()
    for key in ("centroids", "counts", "status", "labels"):
        assert torch.equal(a[key], b[key]), key
    np.testing.assert_allclose(a["inertia"].cpu().numpy(), b["inertia"].cpu().numpy(), rtol=1e-12, atol=0)


# ------------------------------------------------------------------ streaming path (large tasks)

def _sweep_only(wl, flags, want_trace=False, init=None):
    import torch
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                    want_trace=want_trace, flags=flags,
                                    init_centroids=None if init is None else torch.from_numpy(init).to(dw.device))
    torch.cuda.synchronize()
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, init=init, want_labels=True, want_trace=want_trace)
    check_sweep(wl, out, ref, dw.ld)
    return out, ref


@pytest.mark.parametrize("cfg", [1, 2])
def test_streaming_path_on_small_configs(cfg):
    wl = workloads.make_config(cfg, 0)
    wl.n_iter = 12
    _sweep_only(wl, binding.F_STREAMING, want_trace=True)


@pytest.mark.parametrize("d,ks", [(15, (1, 7, 33)), (16, (2, 64, 65)), (31, (5, 100)), (7, (128, 255, 256))])
def test_streaming_path_knob_and_centroid_counts(d, ks):
    wl = workloads.random_task(1200 + d, n=6000, d=d, n_blobs=30, ks=ks, n_iter=5, card_hi=28, sigma=1.4,
                               n_tasks=2, ragged=True)
    _sweep_only(wl, binding.F_STREAMING)


def test_streaming_path_is_the_default_for_large_tasks():
    wl = workloads.random_task(77, n=20000, d=10, n_blobs=20, ks=(4, 40, 90), n_iter=6, card_hi=20)
    out, ref = _sweep_only(wl, 0, want_trace=True)
    # and the vector path (one workgroup per unit) gives the same
    import torch
    dw = binding.DeviceWorkload(wl)
    alt = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                    flags=binding.F_NO_MFMA)
    torch.cuda.synchronize()
    for key in ("centroids", "counts", "labels"):
        assert torch.equal(out[key], alt[key]), key


def test_streaming_path_caller_start_and_exact_ties():
    n, d = 9000, 5
    rows = np.full((n, d), 4, dtype=np.uint8)
    rows[::5, 1] = 7
    wl = workloads.random_task(3, n=8, d=d)
    wl.rows, wl.task_off = rows, np.array([0, n])
    wl.valid = np.ones(n, np.uint8)
    wl.cards = np.full((1, d), 16, np.uint16)
    wl.ks, wl.n_iter = [2], 3
    init = np.zeros((1, 2, d))
    init[0, 0] = 2.0
    init[0, 1] = 6.0
    _sweep_only(wl, binding.F_STREAMING, want_trace=True, init=init)


def test_streaming_path_with_too_few_distinct_rows():
    rng = np.random.default_rng(2)
    base = rng.integers(0, 5, size=(6, 4)).astype(np.uint8)
    rows = base[rng.integers(0, 6, size=5000)]
    wl = workloads.random_task(1, n=8, d=4)
    wl.rows, wl.task_off = np.ascontiguousarray(rows), np.array([0, 5000])
    wl.valid = np.ones(5000, np.uint8)
    wl.cards = np.full((1, 4), 5, np.uint16)
    wl.ks, wl.n_iter = [2, 6, 9], 4
    out, ref = _sweep_only(wl, binding.F_STREAMING)
    assert ref["status"][0, 2] == 1


# ------------------------------------------------------------------ snap / synthesis over row chunks

@pytest.mark.parametrize("seed,d,card_hi,ks", [(501, 7, 6, (8, 24, 60)), (502, 16, 64, (32, 256)),
                                               (503, 3, 3, (2, 5))])
def test_large_tasks_snap_and_synthesis_over_chunks(seed, d, card_hi, ks):
    """Tasks above 16384 rows take the chunked snap and synthesis kernels; invalid rows and a
    well-filled visited set make sure picks are flagged, replaced and dropped."""
    wl = workloads.random_task(seed, n=41001, d=d, card_hi=card_hi, n_blobs=max(ks) // 2 + 1, sigma=1.5,
                               invalid_frac=0.45, ks=ks, n_iter=4, n_visited=30000, n_tasks=3, ragged=True)
    assert np.diff(wl.task_off).max() > 16384
    dw, g, c = run_both(wl)
    check_sweep(wl, g["sweep"], c, dw.ld)
    check_pipeline(wl, g, c)
    flags = c["out_flag"]
    assert (flags == oracle.DROPPED).any() or (flags == oracle.SYNTH).any()


# ------------------------------------------------------------------ sweep that stops at the knee

def _check_knee_sweep(wl, thr, chunk, flags=0):
    """Chunked sweep against the oracle: the chosen k is the one Algorithm 1's loop stops at, every
    computed entry equals the full sweep's, and only whole chunks after the stopping chunk are left out."""
    import torch
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep_knee(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, threshold=thr,
                                         chunk=chunk, want_labels=True, flags=flags, _sfx=dw.sfx)
    torch.cuda.synchronize()
    full = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, want_labels=True)
    loop = oracle.sweep_until_knee(wl.rows, wl.task_off, wl.ks, wl.n_iter, thr)
    chosen = out["chosen"].cpu().numpy()
    status = out["status"].cpu().numpy()
    np.testing.assert_array_equal(chosen, loop["chosen_idx"])
    n_k = len(wl.ks)
    koff = np.concatenate([[0], np.cumsum(wl.ks)])
    cent, cnt = out["centroids"].cpu().numpy(), out["counts"].cpu().numpy()
    inertia, labels = out["inertia"].cpu().numpy(), out["labels"].cpu().numpy()
    for t in range(wl.T):
        # the task stops in the chunk that holds its break (if the loop broke at all)
        broke = loop["ran"][t].sum() > 0 and chosen[t] >= 0 and \
            thr * loop["inertia"][t, chosen[t]] >= _prev_loss(loop, t, chosen[t])
        last_run = min(n_k, (chosen[t] // chunk + 1) * chunk) if broke else n_k
        for ki in range(n_k):
            if ki >= last_run:
                assert status[t, ki] == 3, (t, ki)
                continue
            assert status[t, ki] == full["status"][t, ki], (t, ki)
            if status[t, ki] != 0:
                continue
            sl = slice(koff[ki], koff[ki + 1])
            np.testing.assert_array_equal(cent[t, sl], full["centroids"][t, sl])
            np.testing.assert_array_equal(cnt[t, sl], full["counts"][t, sl])
            np.testing.assert_allclose(inertia[t, ki], full["inertia"][t, ki], rtol=1e-11, atol=0)
            r0, r1 = wl.task_off[t], wl.task_off[t + 1]
            np.testing.assert_array_equal(labels[ki, r0:r1].astype(np.int32), full["labels"][ki, r0:r1])
    return out


def _prev_loss(loop, t, ki):
    prev = np.inf
    for i in range(ki):
        if loop["ran"][t, i]:
            prev = loop["inertia"][t, i]
    return prev


@pytest.mark.parametrize("thr,chunk", [(2.5, 1), (2.5, 4), (1.05, 3), (1.01, 5), (1.0, 64), (1.3, 2)])
def test_knee_sweep_resident_paths(thr, chunk):
    wl = workloads.random_task(900 + chunk, n=1200, d=9, n_blobs=6, ks=tuple(range(1, 20)), n_iter=8, n_tasks=5,
                               ragged=True, card_hi=10)
    _check_knee_sweep(wl, thr, chunk)
    _check_knee_sweep(wl, thr, chunk, flags=binding.F_NO_MFMA)


def test_knee_sweep_with_too_few_distinct_rows_and_an_empty_task():
    wl = workloads.random_task(930, n=40, d=2, card_hi=3, n_blobs=2, ks=(2, 4, 6, 9, 12, 40), n_iter=5, n_tasks=3)
    wl.task_off = np.array([0, 40, 40, 120])             # the middle task has no rows
    _check_knee_sweep(wl, 1.2, 2)


def test_knee_sweep_streaming_path():
    wl = workloads.random_task(940, n=20000, d=10, n_blobs=12, ks=(2, 4, 8, 16, 40, 90), n_iter=5, card_hi=16)
    _check_knee_sweep(wl, 1.3, 2)
    _check_knee_sweep(wl, 2.5, 1)


def test_knee_sweep_on_the_full_model_slice():
    """cfg 5 tasks, the paper's threshold, chunks of 8: nearly every task stops in the first chunk."""
    wl = workloads.make_config(5, 0, scale=4 / 256)
    out = _check_knee_sweep(wl, wl.threshold, 8)
    status = out["status"].cpu().numpy()
    assert (status[:, 8:] == 3).mean() > 0.5


# ------------------------------------------------------------------ visited set as a device table

def _table_for(dw, slots):
    import torch
    table = torch.empty(slots, dtype=torch.int64, device=dw.device)
    binding.cham_visited_table_clear(table)
    ovf = torch.zeros(1, dtype=torch.int32, device=dw.device)
    binding.cham_visited_table_insert_hashes(table, dw.visited, overflow=ovf)
    return table, ovf


def test_synthesis_with_the_visited_table_equals_the_sorted_array():
    import torch
    wl = workloads.make_config(3, 1, scale=8 / 64)
    dw, g, c = run_both(wl)
    table, ovf = _table_for(dw, 1 << 15)
    sy = binding.cham_synthesize_table(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, g["chosen"],
                                       g["snap"]["labels_sel"], g["snap"]["pick_row"], g["snap"]["pick_cfg"], table,
                                       task_salt=wl.salts)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 0
    for key in ("out_cfg", "out_flag", "out_count"):
        np.testing.assert_array_equal(sy[key].cpu().numpy(), c[key])
    # the table holds exactly the visited hashes (the empty mark aside)
    held = table.cpu().numpy().view(np.uint64)
    held = np.sort(held[held != np.uint64(0xFFFFFFFFFFFFFFFF)])
    np.testing.assert_array_equal(held, np.unique(dw.visited_host))


def test_outer_loop_with_a_growing_visited_table():
    """Four rounds of choose k / snap / synthesize on one sweep, with different thresholds; what a
    round returns is inserted into the table and must be treated as visited by the next rounds."""
    import torch
    wl = workloads.make_config(3, 2, scale=6 / 64)
    dw = binding.DeviceWorkload(wl)
    dw.build_visited()
    vis = set(int(v) for v in oracle_visited(wl))
    np.testing.assert_array_equal(np.sort(np.array(sorted(vis), dtype=np.uint64)), np.unique(dw.visited_host))
    table, ovf = _table_for(dw, 1 << 15)
    salts_dev = torch.from_numpy(wl.salts.astype(np.int64)).to(dw.device)
    sw = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter)
    sw_cpu = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    kmax = max(wl.ks)
    grew = 0
    for thr in (1.0, 1.02, 1.3, 2.5, 2.5):
        chosen = binding.cham_select_k(sw["inertia"], sw["status"], thr)
        sn = binding.cham_snap_centroids(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, chosen, sw["centroids"])
        sy = binding.cham_synthesize_table(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, chosen,
                                           sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], table,
                                           task_salt=wl.salts)
        binding.cham_visited_table_insert_configs(table, sy["out_cfg"], dw.d, flags=sy["out_flag"], salts=salts_dev,
                                                  rows_per_salt=kmax, overflow=ovf)
        torch.cuda.synchronize()
        ref = oracle.pipeline(wl, np.array(sorted(vis), dtype=np.uint64), threshold=thr, sweep_out=sw_cpu)
        for key in ("out_cfg", "out_flag", "out_count"):
            np.testing.assert_array_equal(sy[key].cpu().numpy(), ref[key], err_msg=f"{key} at threshold {thr}")
        before = len(vis)
        for t in range(wl.T):
            for cc in range(kmax):
                if ref["out_flag"][t, cc] in (oracle.KEPT, oracle.SYNTH):
                    vis.add(oracle.hash_config(ref["out_cfg"][t, cc], int(wl.salts[t])))
        grew += len(vis) - before
    assert grew > 0 and int(ovf.item()) == 0
    # the last round repeats the threshold of the one before: everything it could return is visited now
    assert (sy["out_flag"].cpu().numpy() != oracle.KEPT).all()


@pytest.mark.parametrize("flags", [0, binding.F_NO_MFMA, binding.F_STREAMING])
def test_warm_start_from_the_previous_round_on_a_changed_sample(flags):
    """Outer loop, next round: the explorer returns a changed sample (here: a third of the rows
    moved by one step in some knobs, a tenth redrawn) and the sweep starts from the centroids the
    previous round ended with.  Some of those centroids may attract no row any more; such a cluster
    keeps its centroid."""
    import torch
    wl = workloads.make_config(3, 1, scale=5 / 64)
    wl.ks, wl.n_iter = [1, 2, 7, 16, 31, 32], 6
    dw = binding.DeviceWorkload(wl)
    first = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, flags=flags)
    first_cpu = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    np.testing.assert_array_equal(first["centroids"].cpu().numpy(), first_cpu["centroids"])
    rng = np.random.default_rng(99)
    rows = wl.rows.astype(np.int64)
    hi = np.repeat(wl.cards.astype(np.int64), np.diff(wl.task_off), axis=0) - 1
    moved = rng.random(rows.shape[0]) < 1 / 3
    rows[moved] += rng.integers(-1, 2, size=(int(moved.sum()), wl.rows.shape[1]))
    redrawn = rng.random(rows.shape[0]) < 0.1
    rows[redrawn] = (rng.random((int(redrawn.sum()), wl.rows.shape[1])) * (hi[redrawn] + 1)).astype(np.int64)
    wl.rows = np.clip(rows, 0, hi).astype(np.uint8)
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, init=first_cpu["centroids"], want_labels=True)
    dw2 = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep(dw2.X, dw2.ld, dw2.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                    init_centroids=first["centroids"], flags=flags)
    torch.cuda.synchronize()
    check_sweep(wl, out, ref, dw2.ld)
    assert (ref["status"] == 0).all()


@pytest.mark.parametrize("flags", [0, binding.F_NO_MFMA, binding.F_STREAMING, binding.F_FORCE_EXACT])
def test_zero_lloyd_steps_is_one_assignment_with_the_start(flags):
    """n_iter = 0: no update at all, labels, counts and loss are those of the starting centroids."""
    wl = workloads.random_task(4242, n=1500, d=11, n_blobs=9, ks=(1, 3, 17, 40), n_iter=0, card_hi=20,
                               n_tasks=3, ragged=True)
    out, ref = _sweep_only(wl, flags, want_trace=True)
    first = oracle.first_distinct(wl.task_rows(0), 40)
    np.testing.assert_array_equal(out["centroids"].cpu().numpy()[0, 21:61], wl.task_rows(0)[first].astype(np.float64))


def test_visited_table_overflow_is_reported_and_lookups_end():
    import torch
    table = torch.empty(4, dtype=torch.int64, device="cuda:0")
    binding.cham_visited_table_clear(table)
    ovf = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    hashes = torch.arange(1, 11, dtype=torch.int64, device="cuda:0") * 7919
    binding.cham_visited_table_insert_hashes(table, hashes, overflow=ovf)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 1
    assert (table.cpu().numpy() != -1).all()             # full
    # a lookup in the full table must terminate: a tiny synthesis call against it
    wl = workloads.random_task(5, n=64, d=3, ks=(2,), n_iter=2)
    dw = binding.DeviceWorkload(wl)
    sw = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter)
    chosen = binding.cham_select_k(sw["inertia"], sw["status"], 2.5)
    sn = binding.cham_snap_centroids(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, chosen, sw["centroids"])
    sy = binding.cham_synthesize_table(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, chosen,
                                       sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], table, task_salt=wl.salts)
    torch.cuda.synchronize()
    assert int(sy["out_count"].sum().item()) >= 0


# ------------------------------------------------------------------ configuration updater

@pytest.mark.parametrize("B,d,steps,card_hi", [(128, 8, 60, 6), (37, 24, 25, 32), (1, 1, 10, 2), (300, 32, 12, 256),
                                               (5, 24, 1300, 16), (3, 31, 1025, 4), (128, 24, 500, 32)])
def test_configuration_updater_matches_the_oracle(B, d, steps, card_hi):
    """Final configurations and the set of distinct configurations reached, against the oracle's walk; the
    step counts span less than one, exactly two and several of the kernel's chunks of steps."""
    import torch
    rng = np.random.default_rng(1000 + B + d)
    cards = rng.integers(1 if d == 1 else 2, card_hi + 1, size=d).astype(np.uint16)
    theta = (rng.random((B, d)) * cards).astype(np.uint8)
    actions = rng.integers(-1, 2, size=(steps, B, d)).astype(np.int8)
    final, order = oracle.update_configs(theta, actions, cards)
    dev = "cuda:0"
    th = torch.from_numpy(theta.copy()).to(dev)
    table = torch.empty(max(1 << 16, 1 << int(np.ceil(np.log2(4 * B * steps)))), dtype=torch.int64, device=dev)
    binding.cham_visited_table_clear(table)
    uniq = torch.zeros((B * steps, d), dtype=torch.uint8, device=dev)
    n_unique = torch.zeros(1, dtype=torch.int32, device=dev)
    ovf = torch.zeros(1, dtype=torch.int32, device=dev)
    # the walk in two calls: the running state (theta, table, list, counter) carries over
    half = steps // 2
    cards_dev = torch.from_numpy(cards.astype(np.int16)).to(dev)
    for a in (actions[:half], actions[half:]):
        binding.cham_update_configs(th, torch.from_numpy(np.ascontiguousarray(a)).to(dev), cards_dev, salt=7,
                                    seen_table=table, unique_rows=uniq, n_unique=n_unique, overflow=ovf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(th.cpu().numpy(), final)
    assert int(ovf.item()) == 0
    n = int(n_unique.item())
    assert n == len(order)
    got = sorted(map(tuple, uniq[:n].cpu().numpy().tolist()))
    assert got == sorted(order)
    # and without bookkeeping
    th2 = torch.from_numpy(theta.copy()).to(dev)
    binding.cham_update_configs(th2, torch.from_numpy(actions).to(dev), cards_dev)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(th2.cpu().numpy(), final)


def test_configuration_updater_reports_a_full_list():
    """A list of distinct configurations shorter than their number: the counter still counts all of them, the
    list holds distinct configurations that were reached, and the overflow word is set."""
    import torch
    rng = np.random.default_rng(5)
    B, d, steps, cap = 16, 12, 700, 100
    cards = rng.integers(8, 33, size=d).astype(np.uint16)
    theta = (rng.random((B, d)) * cards).astype(np.uint8)
    actions = rng.integers(-1, 2, size=(steps, B, d)).astype(np.int8)
    final, order = oracle.update_configs(theta, actions, cards)
    assert len(order) > cap
    dev = "cuda:0"
    th = torch.from_numpy(theta.copy()).to(dev)
    table = torch.empty(1 << 16, dtype=torch.int64, device=dev)
    binding.cham_visited_table_clear(table)
    uniq = torch.full((cap + 8, d), 255, dtype=torch.uint8, device=dev)
    n_unique = torch.zeros(1, dtype=torch.int32, device=dev)
    ovf = torch.zeros(1, dtype=torch.int32, device=dev)
    binding.cham_update_configs(th, torch.from_numpy(actions).to(dev), torch.from_numpy(cards.astype(np.int16)).to(dev),
                                salt=3, seen_table=table, unique_rows=uniq[:cap], n_unique=n_unique, overflow=ovf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(th.cpu().numpy(), final)
    assert int(n_unique.item()) == len(order) and int(ovf.item()) == 1
    rows = uniq.cpu().numpy()
    assert (rows[cap:] == 255).all()                                # nothing written past the capacity
    got = list(map(tuple, rows[:cap].tolist()))
    assert len(set(got)) == cap and set(got) <= set(order)


def test_bench_prints_one_json_line_with_the_contract_fields():
    """bench.py on the smallest workload: one JSON line on stdout carrying the metric, the roofline
    object and the oracle baseline."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--cfg", "2", "--steps", "2", "--warmup", "1",
                        "--knee-chunk", "4", "--no-wide-knobs"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["value"] > 0 and d["unit"] == "evals/s" and "workload" in d["config"]
    rf = d["roofline"]
    assert rf["bound"] in ("hbm", "mfma", "alu") and rf["peak"] > 0 and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]


# ------------------------------------------------------------------ passes really run (stop at the fixed point)

@pytest.mark.parametrize("flags", [0, binding.F_NO_MFMA, binding.F_STREAMING])
def test_passes_run_and_results_of_the_shortened_iteration(flags):
    """The resident kernels stop at the first pass that moves no row; K-means.run of Algorithm 1 with
    its fixed number of steps is what they report.  Checked three ways: against the oracle (which
    runs every pass), against the count of passes the library reports (below the nominal count on
    data that converges, never above it, 0 for a unit with too few distinct rows, nominal on the
    streaming path), and against a second run with just as many steps as the longest unit needed."""
    import torch
    wl = workloads.random_task(4242, n=2500, d=11, n_blobs=5, sigma=0.6, ks=(1, 2, 5, 9, 2400), n_iter=40,
                               n_tasks=2, card_hi=20)
    wl.ks = [1, 2, 5, 9, 64] if flags != binding.F_STREAMING else [1, 2, 5, 9, 200]
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True, flags=flags)
    torch.cuda.synchronize()
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, want_labels=True)
    check_sweep(wl, out, ref, dw.ld)
    passes = binding.cham_sweep_passes(out["workspace"], dw.ld, dw.d, wl.task_off, wl.ks, flags=flags).cpu().numpy()
    status = out["status"].cpu().numpy()
    assert passes.shape == status.shape
    assert (passes[status != 0] == 0).all()
    ok = passes[status == 0]
    assert ok.min() >= 1 and ok.max() <= wl.n_iter + 1
    if flags == binding.F_STREAMING:
        assert (ok == wl.n_iter + 1).all()
    else:
        assert ok.min() < wl.n_iter + 1                    # k = 1 settles in its second pass
        # as many update steps as the longest unit used reproduce every output
        n_short = int(ok.max()) - 1
        again = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, n_short, want_labels=True, flags=flags)
        torch.cuda.synchronize()
        for key in ("status", "counts", "centroids", "labels"):
            assert torch.equal(again[key], out[key]), key
        np.testing.assert_allclose(again["inertia"].cpu().numpy(), out["inertia"].cpu().numpy(), rtol=1e-12, atol=0)
