"""GPU parity for two-byte knobs and up to 64 knobs: the *_u16 entry points through the C ABI against
the CPU oracle, element by element (paper Sec. 2: design spaces are products of the knobs' choice
lists; Sec. 3.3 / Algorithm 1 for what is computed)."""
import numpy as np
import pytest

import oracle
from paper_2001_08743_amd import binding, workloads
from parity_util import check_pipeline, check_sweep, knee_margin, oracle_visited, run_both
from test_gpu_parity import _check_knee_sweep

pytestmark = pytest.mark.gpu


def _full(wl, threshold=None, flags=0):
    assert wl.rows.dtype == np.uint16
    dw, g, c = run_both(wl, threshold=threshold, flags=flags, want_trace=True)
    assert dw.sfx == "_u16"
    check_sweep(wl, g["sweep"], c, dw.ld)
    thr = wl.threshold if threshold is None else threshold
    for t in range(wl.T):
        assert knee_margin(c["inertia"][t], c["status"][t], thr) > 1e-9 or c["inertia"][t].max() == 0
    check_pipeline(wl, g, c)
    return dw, g, c


@pytest.mark.parametrize("seed", [0, 1])
def test_wide_space_whole_path(seed):
    wl = workloads.wide_space(seed, n_tasks=5, n=1800, d=40, ks=range(2, 25), n_iter=10, ragged=True)
    assert wl.rows.max() > 255
    dw, g, c = _full(wl)
    flags = c["out_flag"]
    assert (flags == oracle.SYNTH).any() and (flags == oracle.KEPT).any()


@pytest.mark.parametrize("d", [1, 5, 8, 9, 16, 24, 25, 32, 33, 40, 41, 48, 49, 56, 57, 64])
def test_knob_counts(d):
    wl = workloads.wide_space(10 + d, n_tasks=2, n=900, d=d, ks=(1, 2, 5, 11, 23), n_iter=6, ragged=True,
                              n_visited=512)
    _full(wl, threshold=1.3)


def test_other_thresholds_and_the_exact_flag():
    wl = workloads.wide_space(3, n_tasks=3, n=1200, d=20, ks=range(1, 17), n_iter=8)
    for thr in (1.0, 1.05, 1.5):
        _full(wl, threshold=thr)
    _full(wl, flags=binding.F_FORCE_EXACT)


def test_largest_cardinalities_go_through_knob_windows_of_the_histogram():
    # 16384 choices per knob: the value histogram holds one knob of one cluster at a time
    wl = workloads.wide_space(4, n_tasks=2, n=1500, d=6, ks=(2, 4, 9), n_iter=5, wide_frac=1.0,
                              card_wide=(9000, 16384), n_visited=256)
    assert wl.cards.max() > 12000 and wl.rows.max() > 8000
    _full(wl, threshold=1.2)
    # a mix: small knobs beside one huge one
    wl = workloads.wide_space(5, n_tasks=2, n=1500, d=33, ks=(3, 8), n_iter=5, wide_frac=0.1,
                              card_wide=(16384, 16384), n_visited=256)
    _full(wl, threshold=1.2)


def test_values_up_to_65535_in_sweep_and_snap():
    import torch
    rng = np.random.default_rng(77)
    n, d, k = 3000, 7, 9
    centres = rng.integers(0, 65536, size=(12, d))
    rows = np.clip(centres[rng.integers(0, 12, size=n)] + rng.integers(-400, 401, size=(n, d)), 0, 65535)
    rows[0] = 65535
    rows[1] = 0
    wl = workloads.random_task(1, n=8, d=d)
    wl.rows = rows.astype(np.uint16)
    wl.task_off = np.array([0, n])
    wl.valid = np.ones(n, np.uint8)
    wl.ks, wl.n_iter = [1, 4, k], 7
    dw = binding.DeviceWorkload(wl)
    out = binding.cham_kmeans_sweep_u16(dw.X, dw.ld, d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                        want_trace=True)
    ref = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, want_labels=True, want_trace=True)
    check_sweep(wl, out, ref, dw.ld)
    chosen = torch.tensor([2], dtype=torch.int32, device=dw.device)
    sn = binding.cham_snap_centroids_u16(dw.X, dw.ld, d, wl.task_off, wl.ks, chosen, out["centroids"])
    lab, pick = oracle.snap(wl.rows, ref["centroids"][0, ref["koff"][2]:ref["koff"][2] + k])
    np.testing.assert_array_equal(sn["labels_sel"].cpu().numpy()[:n], lab)
    np.testing.assert_array_equal(sn["pick_row"].cpu().numpy()[0, :k], pick)
    got = binding.knobs_to_host(sn["pick_cfg"])[0, :k]
    for c in range(k):
        if pick[c] >= 0:
            np.testing.assert_array_equal(got[c], wl.rows[pick[c]])
    # a cardinality above 16384 is refused by the synthesis step
    with pytest.raises(binding.ChamError, match="cardinality"):
        binding.cham_synthesize_u16(dw.X, dw.ld, d, wl.task_off, np.full((1, d), 20000), dw.valid, wl.ks, chosen,
                                    sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], None)


def test_byte_valued_data_gives_the_same_results_through_both_families():
    import torch
    wl8 = workloads.make_config(3, 0, scale=4 / 64)
    wl8.ks, wl8.n_iter = list(range(2, 20)), 9
    dw8, g8, c8 = run_both(wl8, want_trace=True)
    wl16 = workloads.make_config(3, 0, scale=4 / 64)
    wl16.ks, wl16.n_iter = list(range(2, 20)), 9
    wl16.rows = wl16.rows.astype(np.uint16)
    wl16.visited_cfg = wl16.visited_cfg.astype(np.uint16)
    dw16, g16, c16 = run_both(wl16, want_trace=True)
    np.testing.assert_array_equal(dw8.visited_host, dw16.visited_host)      # the hashes agree below 256
    for key in ("centroids", "counts", "status", "labels"):
        assert torch.equal(g8["sweep"][key], g16["sweep"][key]), key
    for key in ("inertia", "trace"):        # sums of the same terms in a different order
        np.testing.assert_allclose(g8["sweep"][key].cpu().numpy(), g16["sweep"][key].cpu().numpy(), rtol=1e-12)
    assert torch.equal(g8["chosen"], g16["chosen"])
    for key in ("labels_sel", "pick_row"):
        assert torch.equal(g8["snap"][key], g16["snap"][key]), key
    for part, key in (("snap", "pick_cfg"), ("synth", "out_cfg")):
        np.testing.assert_array_equal(g8[part][key].cpu().numpy(), binding.knobs_to_host(g16[part][key]))
    for key in ("out_flag", "out_count"):
        assert torch.equal(g8["synth"][key], g16["synth"][key]), key
    check_pipeline(wl16, g16, c16)


def test_too_few_distinct_rows_an_empty_task_and_unaligned_offsets():
    rng = np.random.default_rng(5)
    a = rng.integers(0, 3, size=(37, 3)) * 1000          # at most 27 distinct rows
    b = rng.integers(0, 5000, size=(401, 3))
    rows = np.concatenate([a, b]).astype(np.uint16)
    wl = workloads.random_task(2, n=8, d=3)
    wl.rows = rows
    wl.task_off = np.array([0, 37, 37, 438])
    wl.valid = np.ones(438, np.uint8)
    wl.cards = np.full((3, 3), 5000, np.uint16)
    wl.salts = np.arange(3, dtype=np.uint64)
    wl.ks, wl.n_iter = [1, 2, 30, 40], 5
    dw, g, c = _full(wl, threshold=1.5)
    assert c["status"][0, -1] == 1 and (c["status"][1] == 1).all() and (c["status"][2] == 0).all()


def test_knee_sweep_and_the_visited_table():
    import torch
    wl = workloads.wide_space(6, n_tasks=4, n=1000, d=36, ks=range(1, 21), n_iter=6, n_visited=600)
    out = _check_knee_sweep(wl, 2.0, 3)
    dw = binding.DeviceWorkload(wl)
    dw.build_visited()
    # synthesis against a device table filled from configurations equals the sorted-array variant
    sn = binding.cham_snap_centroids_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, out["chosen"], out["centroids"])
    a = binding.cham_synthesize_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, out["chosen"],
                                    sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], dw.visited, task_salt=wl.salts)
    table = torch.empty(1 << 12, dtype=torch.int64, device=dw.device)
    ovf = torch.zeros(1, dtype=torch.int32, device=dw.device)
    binding.cham_visited_table_clear(table)
    binding.cham_visited_table_insert_hashes(table, dw.visited, overflow=ovf)
    b = binding.cham_synthesize_table_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks, out["chosen"],
                                          sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], table, task_salt=wl.salts)
    for key in ("out_cfg", "out_flag", "out_count"):
        assert torch.equal(a[key], b[key]), key
    # what was returned is visited afterwards
    kmax = max(wl.ks)
    salts_dev = torch.from_numpy(wl.salts.astype(np.int64)).to(dw.device)
    binding.cham_visited_table_insert_configs_u16(table, b["out_cfg"], dw.d, flags=b["out_flag"], salts=salts_dev,
                                                  rows_per_salt=kmax, overflow=ovf)
    again = binding.cham_synthesize_table_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.cards, dw.valid, wl.ks,
                                              out["chosen"], sn["labels_sel"], sn["pick_row"], sn["pick_cfg"], table,
                                              task_salt=wl.salts)
    torch.cuda.synchronize()
    assert int(ovf.item()) == 0
    assert (again["out_flag"].cpu().numpy() != oracle.KEPT).all()
    returned = {tuple(r) for r, f in zip(binding.knobs_to_host(b["out_cfg"]).reshape(-1, dw.d),
                                         b["out_flag"].cpu().numpy().reshape(-1)) if f in (oracle.KEPT, oracle.SYNTH)}
    for r, f in zip(binding.knobs_to_host(again["out_cfg"]).reshape(-1, dw.d), again["out_flag"].cpu().numpy().reshape(-1)):
        if f == oracle.SYNTH:
            assert tuple(r) not in returned


def test_a_task_far_larger_than_one_workgroup_pass():
    """40 000 rows in one task: the two-byte path keeps one workgroup per (task, k) and per task in the
    snap and synthesis steps, walking the rows in several passes."""
    wl = workloads.wide_space(8, n_tasks=2, n=40000, d=9, ks=(3, 12, 31), n_iter=5, ragged=True, n_visited=2048)
    assert int(np.diff(wl.task_off).max()) > 16384
    _full(wl, threshold=1.2)


def test_limits_are_reported():
    import torch
    wl = workloads.wide_space(7, n_tasks=1, n=300, d=64, ks=(2, 126), n_iter=2)
    dw = binding.DeviceWorkload(wl)
    with pytest.raises(binding.ChamError, match="bad k list"):
        binding.cham_kmeans_sweep_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter)
    with pytest.raises(binding.ChamError, match="flag"):
        binding.cham_kmeans_sweep_u16(dw.X, dw.ld, dw.d, wl.task_off, [2, 3], wl.n_iter, flags=binding.F_STREAMING)
    # k = 125 at 64 knobs is the largest that fits
    wl.ks = [125]
    out = binding.cham_kmeans_sweep_u16(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True)
    check_sweep(wl, out, oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter, want_labels=True), dw.ld)


# ------------------------------------------------------------------ two-byte knobs on the matrix cores

def _to_device(rows):
    import torch
    n, d = rows.shape
    ld = (n + 63) // 64 * 64
    X = torch.zeros((d, ld), dtype=torch.int16, device="cuda")
    X[:, :n] = torch.from_numpy(np.ascontiguousarray(rows.T).view(np.int16)).cuda()
    return X, ld


@pytest.mark.parametrize("d,n,ks", [(1, 700, (1, 2, 5)), (15, 1500, (3, 33, 64)), (16, 4096, (2, 64)), (31, 3000, (7, 40)),
                                     (32, 2048, (1, 9, 32)), (40, 2048, (2, 17, 32)), (63, 1100, (5, 31)),
                                     (47, 1024, (4, 32)), (33, 130, (3, 6))])
def test_small_valued_two_byte_knobs_on_the_matrix_cores(d, n, ks):
    """Cardinalities of at most 2048: the whole path with the caller's promise (the harness gives it from
    the cardinalities) against the oracle, and the sweep bit for bit against the vector kernel."""
    import torch
    wl = workloads.wide_space(300 + d, n_tasks=3, n=n, d=d, ks=ks, n_iter={47: 0, 31: 1}.get(d, 9), ragged=True, n_visited=256,
                              card_wide=(64, 2048), wide_frac=0.5)
    assert wl.cards.max() <= 2048 and (d < 15 or wl.rows.max() > 255)
    dw, g, c = _full(wl, threshold=1.2)
    v = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                  flags=binding.F_NO_MFMA, _sfx="_u16")
    m = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                  flags=binding.F_VALUES_BELOW_2048, _sfx="_u16")
    torch.cuda.synchronize()
    for key in ("status", "counts", "centroids", "labels"):
        assert torch.equal(v[key], m[key]), key
    np.testing.assert_allclose(m["inertia"].cpu().numpy(), v["inertia"].cpu().numpy(), rtol=1e-12, atol=0)
    passes = binding.cham_sweep_passes(m["workspace"], dw.ld, dw.d, wl.task_off, wl.ks).cpu().numpy()
    assert passes.min() >= 1 and passes.max() <= wl.n_iter + 1
    on_matrix_cores = binding.cham_sweep_path_u16(dw.ld, dw.d, wl.task_off, wl.ks, flags=binding.F_VALUES_BELOW_2048) == 0
    assert on_matrix_cores == (d <= 63 and ((d <= 31 and max(ks) <= 64 and n <= 4096) or (max(ks) <= 32 and n <= 2048)))


@pytest.mark.parametrize("flags", [binding.F_NO_MFMA, binding.F_FORCE_EXACT])
def test_small_valued_two_byte_knobs_on_the_vector_kernel(flags):
    wl = workloads.wide_space(77, n_tasks=4, n=1500, d=40, ks=range(2, 20), n_iter=8, ragged=True, n_visited=512)
    assert wl.cards.max() <= 2048
    _full(wl, threshold=1.2, flags=flags)


def test_a_value_above_the_promised_range_is_reported():
    """CHAM_F_VALUES_BELOW_2048 with a value of 2048 in the rows: every (task, k) reports status 4 and zero
    outputs; without the promise the same rows run on the vector kernel as usual."""
    import torch
    rng = np.random.default_rng(9)
    rows = rng.integers(0, 300, size=(900, 12)).astype(np.uint16)
    rows[517, 3] = 2048
    X, ld = _to_device(rows)
    off = np.array([0, 400, 900], dtype=np.int64)
    ks = [2, 5, 9]
    bad = binding.cham_kmeans_sweep(X, ld, 12, off, ks, 6, want_labels=True, flags=binding.F_VALUES_BELOW_2048,
                                    _sfx="_u16")
    good = binding.cham_kmeans_sweep(X, ld, 12, off, ks, 6, want_labels=True, _sfx="_u16")
    torch.cuda.synchronize()
    assert (bad["status"].cpu().numpy() == 4).all()
    assert float(bad["centroids"].abs().sum().item()) == 0.0 and int(bad["counts"].abs().sum().item()) == 0
    assert (good["status"].cpu().numpy() == 0).all()
    ref = oracle.sweep(rows, off, ks, 6, want_labels=True)
    np.testing.assert_array_equal(good["counts"].cpu().numpy(), ref["counts"])


@pytest.mark.parametrize("d,chunk", [(36, 3), (20, 5)])
def test_knee_sweep_of_small_valued_two_byte_knobs_on_the_matrix_cores(d, chunk):
    """The chunked sweep with the caller's promise: several launches of the matrix-core kernel share one
    packed copy of the rows and one check of the promise."""
    wl = workloads.wide_space(16 + d, n_tasks=4, n=1000, d=d, ks=range(1, 21), n_iter=6, n_visited=300, ragged=True)
    assert wl.cards.max() <= 2048
    ld = (wl.n_total + 63) // 64 * 64
    assert binding.cham_sweep_path_u16(ld, d, wl.task_off, wl.ks, flags=binding.F_VALUES_BELOW_2048) == 0
    _check_knee_sweep(wl, 2.0, chunk, flags=binding.F_VALUES_BELOW_2048)
    _check_knee_sweep(wl, 1.05, chunk, flags=binding.F_VALUES_BELOW_2048)


def test_a_value_above_the_promised_range_is_reported_by_the_knee_sweep():
    import torch
    rng = np.random.default_rng(10)
    rows = rng.integers(0, 500, size=(640, 9)).astype(np.uint16)
    rows[3, 8] = 40000
    X, ld = _to_device(rows)
    off = np.array([0, 640], dtype=np.int64)
    out = binding.cham_kmeans_sweep_knee(X, ld, 9, off, [2, 3, 4, 5], 4, threshold=2.5, chunk=2,
                                         flags=binding.F_VALUES_BELOW_2048, _sfx="_u16")
    torch.cuda.synchronize()
    assert (out["status"].cpu().numpy() == 4).all()
    assert int(out["chosen"].cpu().numpy()[0]) == -1
