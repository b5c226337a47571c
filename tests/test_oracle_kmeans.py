"""Pins for the CPU oracle's k-means sweep (paper Sec. 3.3, Algorithm 1 "K-means.run").

None of these compares the oracle with itself: the references are brute-force
enumeration, closed forms, exact rational arithmetic, invariants, metamorphic
relations and a library Lloyd run (scikit-learn) from the same start.
"""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

import oracle
from paper_2001_08743_amd import workloads


def brute_force_optimum(x, k):
    """Minimum over ALL k-labelings of sum of squared distances to cluster means (exact rationals)."""
    n, d = x.shape
    best = None
    best_lab = None
    for lab in product(range(k), repeat=n):
        cost = Fraction(0)
        for c in range(k):
            idx = [i for i in range(n) if lab[i] == c]
            if not idx:
                continue
            for j in range(d):
                s = sum(int(x[i, j]) for i in idx)
                q = sum(int(x[i, j]) ** 2 for i in idx)
                cost += Fraction(q) - Fraction(s * s, len(idx))
        if best is None or cost < best:
            best, best_lab = cost, lab
    return best, np.array(best_lab)


def start_rows(x, k):
    return x[oracle.first_distinct(x, k)].astype(np.float64)


@pytest.mark.parametrize("seed", range(6))
def test_never_below_brute_force_optimum(seed):
    rng = np.random.default_rng(seed)
    x = rng.integers(0, 6, size=(8, 2)).astype(np.uint8)
    for k in (2, 3):
        if len(oracle.first_distinct(x, k)) < k:
            continue
        jstar, _ = brute_force_optimum(x, k)
        r = oracle.kmeans(x, start_rows(x, k), 20)
        assert r["inertia"] >= float(jstar) - 1e-9


def test_reaches_optimum_on_separated_blobs():
    # three tight groups far apart: Lloyd from one row per group must find the optimum
    x = np.array([[0, 0], [1, 0], [0, 1], [20, 20], [21, 20], [20, 21], [0, 30], [1, 30], [0, 31]],
                 dtype=np.uint8)
    order = [0, 3, 6, 1, 4, 7, 2, 5, 8]          # first three rows: one of each group
    x = x[order]
    jstar, lab = brute_force_optimum(x, 3)
    r = oracle.kmeans(x, start_rows(x, 3), 10)
    assert r["inertia"] == pytest.approx(float(jstar), rel=1e-14)
    # same partition up to naming
    for c in range(3):
        members = np.where(r["labels"] == c)[0]
        assert len(set(lab[members])) == 1


@pytest.mark.parametrize("seed", range(4))
def test_optimal_partition_is_a_fixed_point(seed):
    rng = np.random.default_rng(100 + seed)
    x = rng.integers(0, 9, size=(9, 2)).astype(np.uint8)
    jstar, lab = brute_force_optimum(x, 2)
    if len(set(lab)) < 2:
        pytest.skip("degenerate optimum")
    means = np.stack([x[lab == c].mean(axis=0) for c in range(2)])
    r = oracle.kmeans(x, means, 1)
    # an optimal partition's means cannot be improved by a Lloyd step
    assert r["inertia"] == pytest.approx(float(jstar), rel=1e-12)
    np.testing.assert_allclose(r["mu"], means, rtol=0, atol=1e-12)


@pytest.mark.parametrize("cfg", [1, 2])
def test_k1_closed_form(cfg):
    wl = workloads.make_config(cfg)
    x = wl.task_rows(0)
    r = oracle.kmeans(x, start_rows(x, 1), 3)
    expect = x.shape[0] * np.var(x.astype(np.float64), axis=0).sum()     # N * population variance
    assert r["inertia"] == pytest.approx(expect, rel=1e-12)
    np.testing.assert_allclose(r["mu"][0], x.mean(axis=0), rtol=1e-14)
    assert r["counts"][0] == x.shape[0]


def test_k_equals_distinct_rows_gives_zero_loss():
    rng = np.random.default_rng(7)
    base = rng.integers(0, 5, size=(5, 3)).astype(np.uint8)
    base = np.unique(base, axis=0)
    x = base[rng.integers(0, len(base), size=60)]
    x = np.concatenate([base, x]).astype(np.uint8)
    k = len(base)
    r = oracle.kmeans(x, start_rows(x, k), 5)
    assert r["inertia"] == 0.0
    assert r["counts"].sum() == len(x)


@pytest.mark.parametrize("seed", range(3))
def test_exact_rational_identity_at_convergence(seed):
    wl = workloads.random_task(200 + seed, n=300, d=4, n_blobs=5, sigma=1.0)
    x = wl.task_rows(0)
    k = 5
    r = oracle.kmeans(x, start_rows(x, k), 60)
    lab = r["labels"]
    # converged: every non-empty centroid is the mean of its final members
    for c in range(k):
        if r["counts"][c]:
            np.testing.assert_allclose(r["mu"][c], x[lab == c].mean(axis=0), rtol=0, atol=1e-12)
    total = Fraction(0)
    for c in range(k):
        m = x[lab == c].astype(object)
        if len(m) == 0:
            continue
        for j in range(x.shape[1]):
            s = int(m[:, j].sum())
            total += Fraction(int((m[:, j] ** 2).sum())) - Fraction(s * s, len(m))
    assert r["inertia"] == pytest.approx(float(total), rel=1e-12)


@pytest.mark.parametrize("cfg,k", [(1, 2), (1, 7), (1, 16), (2, 9), (2, 33)])
def test_loss_never_increases_over_lloyd_steps(cfg, k):
    wl = workloads.make_config(cfg)
    x = wl.task_rows(0)
    r = oracle.kmeans(x, start_rows(x, k), 25, want_trace=True)
    tr = r["trace"]
    assert len(tr) == 26
    assert (tr[1:] <= tr[:-1] * (1 + 1e-14)).all()
    assert tr[-1] == r["inertia"]


@pytest.mark.parametrize("cfg", [1, 2])
def test_conservation_of_counts_and_sums(cfg):
    wl = workloads.make_config(cfg)
    x = wl.task_rows(0)
    sw = oracle.sweep(wl.rows, wl.task_off, wl.ks, 4, want_labels=True)
    for ki, k in enumerate(wl.ks):
        cnt = sw["counts"][0, sw["koff"][ki]:sw["koff"][ki] + k]
        assert cnt.sum() == x.shape[0]
        lab = sw["labels"][ki]
        assert lab.min() >= 0 and lab.max() < k
        np.testing.assert_array_equal(np.bincount(lab, minlength=k), cnt)


def test_sweep_start_is_prefix_of_first_distinct_rows():
    wl = workloads.make_config(1)
    x = wl.task_rows(0)
    sw = oracle.sweep(wl.rows, wl.task_off, wl.ks, 0)      # zero Lloyd steps: centroids = start
    first = oracle.first_distinct(x, max(wl.ks))
    assert len(np.unique(x[first], axis=0)) == len(first)
    # rows skipped before each taken row are duplicates of an earlier taken row
    taken = []
    for i in range(first[-1] + 1):
        if any((x[i] == x[q]).all() for q in taken):
            assert i not in first
        else:
            taken.append(i)
    assert taken == list(first)
    for ki, k in enumerate(wl.ks):
        np.testing.assert_array_equal(sw["centroids"][0, sw["koff"][ki]:sw["koff"][ki] + k], x[first[:k]])


def test_too_few_distinct_rows_sets_status():
    x = np.array([[1, 1], [1, 1], [2, 2], [1, 1], [2, 2]], dtype=np.uint8)
    sw = oracle.sweep(x, [0, 5], [1, 2, 3], 3)
    assert list(sw["status"][0]) == [0, 0, 1]
    assert sw["inertia"][0, 2] == 0.0
    assert sw["inertia"][0, 1] == 0.0
    assert (sw["counts"][0, 3:] == 0).all()


def test_metamorphic_duplicate_rows():
    wl = workloads.random_task(11, n=200, d=5, n_blobs=4)
    x = wl.task_rows(0)
    k = 4
    a = oracle.kmeans(x, start_rows(x, k), 30)
    x2 = np.repeat(x, 2, axis=0)
    b = oracle.kmeans(x2, start_rows(x2, k), 30)
    np.testing.assert_allclose(b["mu"], a["mu"], rtol=0, atol=1e-12)
    assert b["inertia"] == pytest.approx(2 * a["inertia"], rel=1e-13)
    np.testing.assert_array_equal(b["counts"], 2 * a["counts"])


def test_metamorphic_shift_and_column_swap():
    # well separated blobs so that no label sits on a rounding-sensitive tie
    rng = np.random.default_rng(5)
    centres = np.array([[2, 2, 2], [12, 2, 9], [2, 12, 5], [12, 12, 12]])
    x = (centres[rng.integers(0, 4, size=240)] + rng.integers(-1, 2, size=(240, 3))).astype(np.uint8)
    k = 4
    a = oracle.kmeans(x, start_rows(x, k), 20)
    shifted = x.copy()
    shifted[:, 1] += 7
    b = oracle.kmeans(shifted, start_rows(shifted, k), 20)
    np.testing.assert_array_equal(a["labels"], b["labels"])
    assert b["inertia"] == pytest.approx(a["inertia"], rel=1e-12)
    swapped = x[:, [2, 1, 0]].copy()
    c = oracle.kmeans(swapped, start_rows(swapped, k), 20)
    np.testing.assert_array_equal(a["labels"], c["labels"])
    np.testing.assert_allclose(c["mu"][:, [2, 1, 0]], a["mu"], rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed,k,n_iter", [(0, 3, 4), (1, 5, 7), (2, 8, 40), (3, 6, 2)])
def test_against_library_lloyd(seed, k, n_iter):
    """scikit-learn's Lloyd from the same start, same number of steps (cases without empty clusters)."""
    sklearn_cluster = pytest.importorskip("sklearn.cluster")
    wl = workloads.random_task(300 + seed, n=500, d=6, n_blobs=k, sigma=1.2, card_hi=20)
    x = wl.task_rows(0)
    # Start rows nudged off the integer grid: from integer centroids many rows sit at exactly equal
    # distances, and the library breaks such ties by the rounding of its expanded distance formula
    # rather than by lowest index.  Off the grid there are no exact ties and both must agree.
    rng = np.random.default_rng(seed)
    init = start_rows(x, k) + rng.uniform(-0.3, 0.3, size=(k, x.shape[1]))
    r = oracle.kmeans(x, init, n_iter)
    if (r["counts"] == 0).any():
        pytest.skip("library relocates empty clusters; rule differs by design")
    import warnings
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        km = sklearn_cluster.KMeans(n_clusters=k, init=init, n_init=1, algorithm="lloyd",
                                    max_iter=n_iter, tol=0.0).fit(x.astype(np.float64))
    np.testing.assert_allclose(r["mu"], km.cluster_centers_, rtol=1e-11, atol=1e-11)
    assert r["inertia"] == pytest.approx(km.inertia_, rel=1e-11)
    np.testing.assert_array_equal(r["labels"], km.labels_)


def test_empty_cluster_keeps_its_centroid():
    # caller-supplied start with one centroid far from all rows: it never gets a member
    x = np.array([[0, 0], [0, 1], [1, 0], [9, 9], [9, 8]], dtype=np.uint8)
    init = np.array([[0.0, 0.0], [9.0, 9.0], [200.0, 200.0]])
    r = oracle.kmeans(x, init, 5)
    assert r["counts"][2] == 0
    np.testing.assert_array_equal(r["mu"][2], [200.0, 200.0])
    np.testing.assert_allclose(r["mu"][0], [1 / 3, 1 / 3], rtol=1e-15)


def test_tie_goes_to_lowest_cluster():
    # row (1) sits exactly between centroids 0 and 2 -> label 0 ... and between equal centroids
    x = np.array([[1], [0], [2]], dtype=np.uint8)
    init = np.array([[0.0], [2.0]])
    r = oracle.kmeans(x, init, 0)
    assert list(r["labels"]) == [0, 0, 1]


def test_batch_equals_single_tasks():
    wl = workloads.random_task(21, n=180, d=5, n_tasks=3, ragged=True, ks=(2, 4, 5), n_iter=6)
    sw = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    for t in range(wl.T):
        x = wl.task_rows(t)
        for ki, k in enumerate(wl.ks):
            r = oracle.kmeans(x, start_rows(x, k), wl.n_iter)
            np.testing.assert_array_equal(sw["centroids"][t, sw["koff"][ki]:sw["koff"][ki] + k], r["mu"])
            assert sw["inertia"][t, ki] == r["inertia"]


# ------------------------------------------------------------------ the loop that stops at the knee

@pytest.mark.parametrize("seed,thr", [(11, 2.5), (12, 1.05), (13, 1.01), (14, 1.0), (15, 1.3)])
def test_early_break_loop_agrees_with_full_sweep_then_select(seed, thr):
    """Algorithm 1 run literally (k after k, break at the knee) must pick the k that the knee rule
    picks on the full loss curve, and every k it ran must give the full sweep's result."""
    from paper_2001_08743_amd import workloads
    wl = workloads.random_task(seed, n=300, d=5, n_blobs=5, ks=(1, 2, 3, 4, 6, 8, 11), n_iter=8, n_tasks=3,
                               ragged=True, card_hi=6)
    full = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    eb = oracle.sweep_until_knee(wl.rows, wl.task_off, wl.ks, wl.n_iter, thr)
    koff = np.concatenate([[0], np.cumsum(wl.ks)])
    for t in range(wl.T):
        want = oracle.select_k(full["inertia"][t], full["status"][t], thr)
        assert eb["chosen_idx"][t] == want
        # nothing after the break was run, everything usable before it was
        assert not eb["ran"][t, want + 1:].any()
        for ki in range(want + 1):
            assert eb["ran"][t, ki] == (full["status"][t, ki] == 0)
            if eb["ran"][t, ki]:
                assert eb["inertia"][t, ki] == full["inertia"][t, ki]
                np.testing.assert_array_equal(eb["centroids"][t][ki], full["centroids"][t, koff[ki]:koff[ki + 1]])
                np.testing.assert_array_equal(eb["counts"][t][ki], full["counts"][t, koff[ki]:koff[ki + 1]])


def test_early_break_loop_hand_case():
    """Two well separated pairs of points: loss(1) = 8, loss(2) = 0.5 * 4 = ... computed by hand below."""
    rows = np.array([[0], [1], [10], [11]], dtype=np.uint8)
    # k=1: mean 5.5, loss = 5.5^2 + 4.5^2 + 4.5^2 + 5.5^2 = 101; k=2 from starts {0, 1}: converges to
    # {0.5, 10.5}, loss = 4 * 0.25 = 1; k=3 from starts {0, 1, 10}: {0}, {1}, {10, 11}: loss = 0.5
    eb = oracle.sweep_until_knee(rows, [0, 4], [1, 2, 3], 10, threshold=1.5)
    np.testing.assert_allclose(eb["inertia"][0], [101.0, 1.0, 0.5])
    assert eb["chosen_idx"][0] == 2 and eb["ran"][0].all()          # 1.5 * 0.5 = 0.75 < 1: no break, last k
    eb = oracle.sweep_until_knee(rows, [0, 4], [1, 2, 3], 10, threshold=2.5)
    assert eb["chosen_idx"][0] == 2                                  # 2.5 * 0.5 = 1.25 >= 1: break at k = 3
    eb = oracle.sweep_until_knee(rows, [0, 4], [1, 2, 3], 10, threshold=150.0)
    assert eb["chosen_idx"][0] == 1 and not eb["ran"][0, 2]          # 150 * 1 >= 101: break at k = 2
