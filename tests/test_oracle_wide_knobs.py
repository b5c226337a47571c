"""Pins for the CPU oracle on knob values above 255 and more than 32 knobs (paper Sec. 2: a knob's
list of choices, e.g. the split factors of a loop, can have hundreds of entries).

As in the other oracle pin files nothing here compares the oracle with itself: the references are
brute-force enumeration and closed forms in exact rationals, metamorphic relations whose truth does
not depend on the implementation, and hand-worked cases.  Every case would fail if a value were cut
to its low byte anywhere on the way.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from test_oracle_kmeans import brute_force_optimum, start_rows
from test_oracle_select_synth import H, vis

KEPT, SYNTH, DROPPED, EMPTY = oracle.KEPT, oracle.SYNTH, oracle.DROPPED, oracle.EMPTY


@pytest.mark.parametrize("seed", range(4))
def test_never_below_brute_force_optimum_with_wide_values(seed):
    rng = np.random.default_rng(100 + seed)
    x = (rng.integers(0, 6, size=(8, 2)) * 9000 + rng.integers(0, 300, size=(8, 2))).astype(np.uint16)
    for k in (2, 3):
        jstar, _ = brute_force_optimum(x, k)
        r = oracle.kmeans(x, start_rows(x, k), 20)
        assert r["inertia"] >= float(jstar) * (1 - 1e-12)


def test_reaches_optimum_on_separated_blobs_that_differ_only_above_the_low_byte():
    # the three groups have equal low bytes; only the high byte tells them apart
    base = np.array([[0, 0], [1, 0], [0, 1]])
    x = np.concatenate([base, base + [256 * 20, 256 * 3], base + [256 * 7, 256 * 90]]).astype(np.uint16)
    x = x[[0, 3, 6, 1, 4, 7, 2, 5, 8]]
    jstar, lab = brute_force_optimum(x, 3)
    r = oracle.kmeans(x, start_rows(x, 3), 10)
    assert r["inertia"] == pytest.approx(float(jstar), rel=1e-14)
    for c in range(3):
        assert len(set(lab[np.where(r["labels"] == c)[0]])) == 1


@pytest.mark.parametrize("d", [3, 40, 64])
def test_k1_closed_form_in_exact_rationals(d):
    rng = np.random.default_rng(d)
    x = rng.integers(0, 65536, size=(57, d)).astype(np.uint16)
    r = oracle.kmeans(x, start_rows(x, 1), 3)
    n = x.shape[0]
    want = Fraction(0)
    for j in range(d):
        col = [int(v) for v in x[:, j]]
        want += Fraction(sum(v * v for v in col)) - Fraction(sum(col) ** 2, n)
        assert r["mu"][0, j] == pytest.approx(sum(col) / n, rel=1e-15)
    assert r["inertia"] == pytest.approx(float(want), rel=1e-12)
    assert r["counts"][0] == n


def test_rows_that_differ_only_in_the_high_byte_are_distinct():
    x = np.array([[1, 5], [257, 5], [1, 5], [1, 5 + 512], [257, 5]], dtype=np.uint16)
    np.testing.assert_array_equal(oracle.first_distinct(x, 5), [0, 1, 3])
    r = oracle.kmeans(x, start_rows(x, 3), 4)
    assert r["inertia"] == 0.0
    np.testing.assert_array_equal(r["labels"], [0, 1, 0, 2, 1])
    sw = oracle.sweep(x, [0, 5], [3, 4], 2)
    np.testing.assert_array_equal(sw["status"], [[0, 1]])


def test_shift_across_the_byte_boundary_changes_nothing():
    rng = np.random.default_rng(8)
    centres = np.array([[2, 2, 2], [12, 2, 9], [2, 12, 5], [12, 12, 12]])
    x = (centres[rng.integers(0, 4, size=240)] + rng.integers(-1, 2, size=(240, 3))).astype(np.uint16)
    a = oracle.kmeans(x, start_rows(x, 4), 20)
    shifted = x.copy()
    shifted[:, 1] += 250            # values now straddle 255
    shifted[:, 2] += 40000
    b = oracle.kmeans(shifted, start_rows(shifted, 4), 20)
    np.testing.assert_array_equal(a["labels"], b["labels"])
    assert b["inertia"] == pytest.approx(a["inertia"], rel=1e-12)
    np.testing.assert_allclose(b["mu"] - [0, 250, 40000], a["mu"], rtol=0, atol=1e-9)


def test_scaling_every_knob_scales_the_loss_by_the_square():
    rng = np.random.default_rng(9)
    centres = np.array([[2, 2], [12, 2], [2, 12], [12, 12]])
    x = (centres[rng.integers(0, 4, size=200)] + rng.integers(-1, 2, size=(200, 2))).astype(np.uint16)
    a = oracle.kmeans(x, start_rows(x, 4), 15)
    big = (x.astype(np.int64) * 4096).astype(np.uint16)      # a power of two: every operation scales exactly
    b = oracle.kmeans(big, start_rows(big, 4), 15)
    np.testing.assert_array_equal(a["labels"], b["labels"])
    assert b["inertia"] == a["inertia"] * 4096.0 ** 2
    np.testing.assert_array_equal(b["mu"], a["mu"] * 4096.0)


def test_snap_and_mode_hand_worked_with_wide_values():
    x = np.array([[300, 7], [300, 9], [1000, 9], [7, 9], [300, 1000], [60000, 60000]], dtype=np.uint16)
    mu = np.array([[400.0, 10.0], [59990.0, 60010.0]])
    lab, pick = oracle.snap(x, mu)
    np.testing.assert_array_equal(lab, [0, 0, 0, 0, 0, 1])
    # squared distances to (400, 10): 10009, 10001, 360001, 154450, 990100 -> row 1
    np.testing.assert_array_equal(pick, [1, 5])
    cards = [65535, 65535]
    # the pick (300, 9) is visited: per-knob mode of cluster 0 is (300, 9) again -> visited -> dropped
    cfg, flag, cnt = oracle.synthesize(x, cards, None, lab, pick, vis([300, 9]), 0)
    assert list(flag) == [DROPPED, KEPT] and cnt == 1
    np.testing.assert_array_equal(cfg, [[0, 0], [60000, 60000]])
    # with row 1 invalid (so its pick is flagged) the valid members are (300,7) (1000,9) (7,9) (300,1000):
    # knob 0 -> 300 (twice), knob 1 -> 9 (twice)
    valid = [1, 0, 1, 1, 1, 1]
    cfg, flag, cnt = oracle.synthesize(x, cards, valid, lab, pick, np.zeros(0, np.uint64), 0)
    assert list(flag) == [SYNTH, KEPT] and cnt == 2
    np.testing.assert_array_equal(cfg, [[300, 9], [60000, 60000]])
    # a tie between 300 and 7 in knob 0 goes to the smaller value
    x2 = np.array([[300, 1], [7, 1], [300, 1], [7, 1]], dtype=np.uint16)
    cfg, flag, cnt = oracle.synthesize(x2, [400, 2], [0, 1, 1, 1], [0, 0, 0, 0], [0], np.zeros(0, np.uint64), 0)
    assert list(flag) == [SYNTH] and list(cfg[0]) == [7, 1]


def test_hash_of_wide_values():
    # one xor-multiply step per knob, the whole value in the step (Python integers, independent code)
    for cfg, salt in (([300], 0), ([65535, 0, 256], 5), ([255, 256, 257, 40000], 123456789)):
        assert oracle.hash_config(cfg, salt) == H(cfg, salt)
    # multiplication by an odd constant is a bijection: one-knob configurations never collide
    h = oracle.hash_rows(np.arange(65536, dtype=np.uint16).reshape(-1, 1), 3)
    assert len(np.unique(h)) == 65536
    # the pair (1, 0) is not the single value 256, nor the single value 1
    assert len({oracle.hash_config([1, 0]), oracle.hash_config([256]), oracle.hash_config([1])}) == 3
