"""GPU parity over the full byte range of knob values and on inputs built to stress the error bound of
the f16 matrix-core screens: every knob takes values 0..255 (a knob's choice list, Sec. 2.2, may have
up to 256 entries on the byte path), centroids sit far from the centring offset, and many rows lie
(almost) halfway between two centroids.  Every case is compared with the CPU oracle and, for the
sweep, with the library's own all-double path (CHAM_F_FORCE_EXACT)."""
import numpy as np
import pytest

import oracle
from paper_2001_08743_amd import binding, workloads
from parity_util import check_pipeline, check_sweep, run_both

pytestmark = pytest.mark.gpu


def _wl(rows, sizes, cards, ks, n_iter, n_visited=64, valid=None, seed=0):
    """A workload from explicit rows (no blobs drawn here)."""
    rows = np.ascontiguousarray(rows, dtype=np.uint8)
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    wl = workloads.random_task(seed, n=8, d=rows.shape[1])
    wl.rows, wl.task_off = rows, off
    wl.valid = np.ones(len(rows), np.uint8) if valid is None else np.ascontiguousarray(valid, dtype=np.uint8)
    wl.cards = np.ascontiguousarray(cards, dtype=np.uint16).reshape(len(sizes), rows.shape[1])
    wl.ks, wl.n_iter = list(ks), n_iter
    wl.salts = np.arange(len(sizes), dtype=np.uint64)
    rng = np.random.default_rng(seed + 77)
    nv = min(n_visited, len(rows))
    pick = rng.choice(len(rows), size=nv, replace=False)
    wl.visited_cfg = rows[pick].copy()
    task_of_row = np.repeat(np.arange(len(sizes)), sizes)
    wl.visited_task = task_of_row[pick].astype(np.int64)
    wl.visited_raw = rng.integers(0, 2 ** 63, size=n_visited, dtype=np.uint64)
    wl.n_visited = n_visited
    return wl


def _both_and_exact(wl, threshold=1.05, flags=0):
    import torch
    dw, g, c = run_both(wl, threshold=threshold, flags=flags)
    check_sweep(wl, g["sweep"], c, dw.ld)
    check_pipeline(wl, g, c)
    ex = binding.cham_kmeans_sweep(dw.X, dw.ld, dw.d, wl.task_off, wl.ks, wl.n_iter, want_labels=True,
                                   flags=binding.F_FORCE_EXACT)
    torch.cuda.synchronize()
    for key in ("status", "counts", "centroids", "labels"):
        assert torch.equal(ex[key], g["sweep"][key]), key
    return dw, g, c


def _blobs_255(rng, n, d, n_blobs, sigma):
    centres = rng.uniform(0, 255, size=(n_blobs, d))
    which = rng.integers(0, n_blobs, size=n)
    x = np.rint(centres[which] + sigma * rng.standard_normal((n, d)))
    return np.clip(x, 0, 255).astype(np.uint8)


@pytest.mark.parametrize("d", [13, 16, 29, 31])
def test_byte_values_0_to_255_resident_matrix_core(d):
    rng = np.random.default_rng(1000 + d)
    sizes = [4096, 1500]
    rows = np.concatenate([_blobs_255(rng, n, d, 20, 9.0) for n in sizes])
    rows[:8] = 0
    rows[8:16] = 255                       # the corners of the value range are present
    valid = (rng.random(len(rows)) > 0.05).astype(np.uint8)
    wl = _wl(rows, sizes, np.full((2, d), 256), ks=(1, 2, 7, 16, 33, 64), n_iter=12, valid=valid, seed=d)
    assert binding.cham_sweep_path((len(rows) + 63) // 64 * 64, d, wl.task_off, wl.ks) == 0
    _both_and_exact(wl)


@pytest.mark.parametrize("d", [16, 31])
def test_byte_values_0_to_255_streaming_k_256(d):
    rng = np.random.default_rng(2000 + d)
    sizes = [9000]
    rows = _blobs_255(rng, sizes[0], d, 150, 6.0)
    rows[:4] = 0
    rows[4:8] = 255
    wl = _wl(rows, sizes, np.full((1, d), 256), ks=(64, 200, 256), n_iter=6, seed=d)
    assert binding.cham_sweep_path((len(rows) + 63) // 64 * 64, d, wl.task_off, wl.ks) == 1
    _both_and_exact(wl, threshold=1.01)


def test_uniform_random_bytes_cardinality_256_snap_and_synthesis():
    """No cluster structure at all: every knob uniform over 0..255, a third of the rows invalid, half of the
    rows visited, so that picks are flagged and the per-knob mode runs over 256-bin histograms."""
    rng = np.random.default_rng(31)
    d, sizes = 24, [2048, 700, 3]
    rows = rng.integers(0, 256, size=(sum(sizes), d)).astype(np.uint8)
    rows[100:160] = rows[100]              # a block of duplicates: a mode that is not a tie
    valid = (rng.random(len(rows)) > 0.33).astype(np.uint8)
    wl = _wl(rows, sizes, np.full((3, d), 256), ks=(1, 2, 3, 9, 40), n_iter=8, n_visited=1400, valid=valid, seed=5)
    dw, g, c = _both_and_exact(wl, threshold=1.0)
    flags = g["synth"]["out_flag"].cpu().numpy()
    assert (flags == binding.OUT_SYNTH).any() or (flags == binding.OUT_DROPPED).any()


@pytest.mark.parametrize("flags", [0, binding.F_STREAMING])
def test_near_ties_far_from_the_centring_offset(flags):
    """Rows on (and next to) the bisecting planes of centroids that sit in opposite corners of the value
    range: the scores are as large as they get (|x'| and |mu'| near 128 per knob after centring) while the
    gaps between the best two are zero or a few units in the last place of the fp32 screen."""
    rng = np.random.default_rng(77)
    d = 29
    n_c = 12
    # centroids-to-be: corner-ish points, each a block of identical rows so that they are the first distinct rows
    corners = (rng.integers(0, 2, size=(n_c, d)) * 255).astype(np.int64)
    corners[:, :3] = rng.integers(0, 256, size=(n_c, 3))
    blocks = [np.repeat(corners[i:i + 1], 40, axis=0) for i in range(n_c)]
    # midpoints of centroid pairs (exact ties when the coordinate sums are even) and their neighbours
    mids = []
    for a in range(n_c):
        for b in range(a + 1, n_c):
            m = (corners[a] + corners[b]) // 2
            for dj in (-1, 0, 1):
                v = m.copy()
                v[rng.integers(0, d)] += dj
                mids.append(np.clip(v, 0, 255))
    fill = rng.integers(0, 256, size=(1500, d))
    body = np.concatenate([np.array(mids), fill])
    rng.shuffle(body)
    rows = np.concatenate([np.concatenate(blocks), body]).astype(np.uint8)
    sizes = [len(rows)]
    wl = _wl(rows, sizes, np.full((1, d), 256), ks=(2, 5, n_c), n_iter=9, seed=9)
    _both_and_exact(wl, threshold=1.01, flags=flags)


def test_two_value_knobs_with_values_0_and_255_only():
    """Every knob is 0 or 255: the largest possible spread per knob, exact ties everywhere."""
    rng = np.random.default_rng(4)
    d = 16
    rows = (rng.integers(0, 2, size=(3000, d)) * 255).astype(np.uint8)
    wl = _wl(rows, [3000], np.full((1, d), 256), ks=(1, 2, 4, 8, 31, 64), n_iter=10, seed=2)
    _both_and_exact(wl)
