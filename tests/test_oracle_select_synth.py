"""Pins for the oracle's knee selection, snap, Sample Synthesis, dedupe and hash
(paper Algorithm 1 and Sec. 3.3).  Expected values are worked by hand or come
from the published FNV-1a vectors; none is produced by the oracle.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import DROPPED, EMPTY, KEPT, SYNTH


def read_golden(golden_dir, name):
    out = {}
    with open(os.path.join(golden_dir, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split()
            out[key] = val
    return out


# ---------------------------------------------------------------- knee (Algorithm 1, first loop)

def test_paper_threshold_value(golden_dir):
    g = read_golden(golden_dir, "paper_hyperparameters.txt")
    assert float(g["threshold_meta"]) == 2.5


def test_knee_stops_where_the_loss_stops_dropping_fast():
    # 2.5*30 = 75 < 100: no stop at index 1; 2.5*20 = 50 >= 30: stop at index 2
    assert oracle.select_k([100, 30, 20, 19], None, 2.5) == 2


def test_knee_hand_curves():
    # previous_loss starts at infinity: index 0 can never stop the loop
    assert oracle.select_k([5.0], None, 2.5) == 0
    assert oracle.select_k([0.0, 0.0], None, 2.5) == 1          # 2.5*0 >= 0
    # equality counts (">=")
    assert oracle.select_k([100, 50], None, 2.0) == 1
    assert oracle.select_k([100, 49.999, 30], None, 2.0) == 2   # 99.998 < 100 ; 60 >= 49.999
    # a curve that drops 3x at every step never satisfies 2.5*L >= prev: last index
    assert oracle.select_k([81, 27, 9, 3], None, 2.5) == 3
    # typical slowly decreasing curve: the second k already stops (2.5*90 >= 100)
    assert oracle.select_k([100, 90, 80, 70], None, 2.5) == 1
    # threshold 1: stops only when the loss fails to decrease
    assert oracle.select_k([10, 9, 8, 8, 7], None, 1.0) == 3
    assert oracle.select_k([10, 9, 8, 7.5, 7], None, 1.0) == 4


def test_knee_skips_unusable_entries():
    # entries with non-zero status are treated as absent
    assert oracle.select_k([100, 0, 30, 20], [0, 1, 0, 0], 2.5) == 3   # 75 < 100 ; 50 >= 30
    assert oracle.select_k([100, 90, 0], [0, 0, 1], 2.5) == 1
    assert oracle.select_k([100, 30, 0, 0], [0, 0, 1, 1], 2.5) == 1    # no stop: last usable
    assert oracle.select_k([0, 0], [1, 1], 2.5) == -1


# ---------------------------------------------------------------- snap

def test_snap_hand_worked_1d():
    # clusters {0,1,2,3} around 1.5 and {10,11} around 10.5
    x = np.array([[3], [10], [0], [2], [1], [11]], dtype=np.uint8)
    mu = np.array([[1.5], [10.5]])
    lab, pick = oracle.snap(x, mu)
    assert list(lab) == [0, 1, 0, 0, 0, 1]
    # members at distance 0.5 from 1.5: rows 3 (value 2) and 4 (value 1): exact tie -> smaller row
    assert pick[0] == 3
    # rows 1 and 5 tie around 10.5 -> row 1
    assert pick[1] == 1


def test_snap_hand_worked_2d_and_empty_cluster():
    x = np.array([[0, 0], [4, 4], [1, 1], [5, 5], [4, 5]], dtype=np.uint8)
    mu = np.array([[0.75, 0.75], [4.25, 4.75], [100.0, 100.0]])
    lab, pick = oracle.snap(x, mu)
    assert list(lab) == [0, 1, 0, 1, 1]
    assert pick[0] == 2          # (1,1): 0.125 < (0,0): 1.125
    assert pick[1] == 4          # (4,5): 0.125 ; (4,4): 0.625 ; (5,5): 0.625
    assert pick[2] == -1


# ---------------------------------------------------------------- hash

def test_hash_matches_published_fnv1a_vectors(golden_dir):
    g = read_golden(golden_dir, "fnv1a64_vectors.txt")
    for s, digest in g.items():
        data = b"" if s == "EMPTY" else s.encode("ascii")
        cfg = np.frombuffer(data, dtype=np.uint8) if data else np.zeros(0, np.uint8)
        assert oracle.hash_config(cfg, 0) == int(digest, 16), s


def test_hash_salt_is_mixed_into_the_basis():
    # salt s: basis ^ (s * 0x9E3779B97F4A7C15 mod 2^64), then the same byte steps (big-int arithmetic)
    M = 1 << 64
    for salt, cfg in [(1, [1, 2]), (7, [0]), (255, [3, 1, 4, 1, 5])]:
        h = 0xCBF29CE484222325 ^ ((salt * 0x9E3779B97F4A7C15) % M)
        for v in cfg:
            h = ((h ^ v) * 0x100000001B3) % M
        assert oracle.hash_config(np.array(cfg, dtype=np.uint8), salt) == h
    a = oracle.hash_config(np.array([1, 2, 3], dtype=np.uint8), 0)
    b = oracle.hash_config(np.array([1, 2, 3], dtype=np.uint8), 1)
    assert a != b


def test_hash_rows_per_row_salts():
    x = np.array([[1, 2], [1, 2], [3, 4]], dtype=np.uint8)
    h = oracle.hash_rows(x, np.array([0, 5, 5], dtype=np.uint64))
    assert h[0] == oracle.hash_config(x[0], 0)
    assert h[1] == oracle.hash_config(x[1], 5)
    assert h[2] == oracle.hash_config(x[2], 5)


# ---------------------------------------------------------------- synthesis + dedupe

def H(cfg, salt=0):
    """FNV-1a with the salt mix, in Python integers (independent of the oracle)."""
    M = 1 << 64
    h = 0xCBF29CE484222325 ^ ((salt * 0x9E3779B97F4A7C15) % M)
    for v in cfg:
        h = ((h ^ int(v)) * 0x100000001B3) % M
    return h


def vis(*cfgs, salt=0):
    return np.array(sorted(H(c, salt) for c in cfgs), dtype=np.uint64)


def test_unvisited_valid_picks_pass_through():
    x = np.array([[0, 0], [0, 1], [5, 5], [5, 4]], dtype=np.uint8)
    cards = [8, 8]
    lab = [0, 0, 1, 1]
    cfg, flag, cnt = oracle.synthesize(x, cards, None, lab, [1, 2], vis([7, 7]), 0)
    assert list(flag) == [KEPT, KEPT] and cnt == 2
    np.testing.assert_array_equal(cfg, [[0, 1], [5, 5]])


def test_visited_pick_replaced_by_per_knob_mode():
    # cluster 0 members: (1,3) (1,4) (2,4) (1,3) (2,3)  -> knob0 mode 1 (3x), knob1 mode 3 (3x)
    x = np.array([[1, 3], [1, 4], [2, 4], [1, 3], [2, 3], [7, 7]], dtype=np.uint8)
    lab = [0, 0, 0, 0, 0, 1]
    # the pick (2,4) is visited; the mode (1,3) is not
    cfg, flag, cnt = oracle.synthesize(x, [8, 8], None, lab, [2, 5], vis([2, 4]), 0)
    assert list(flag) == [SYNTH, KEPT] and cnt == 2
    np.testing.assert_array_equal(cfg, [[1, 3], [7, 7]])


def test_mode_tie_takes_smallest_value_and_ignores_invalid_rows():
    # knob0 values among valid members: 4,4,2,2 -> tie -> 2 ; the invalid rows hold 6,6,6 (would win)
    x = np.array([[4, 1], [4, 1], [2, 1], [2, 0], [6, 0], [6, 0], [6, 0]], dtype=np.uint8)
    valid = [1, 1, 1, 1, 0, 0, 0]
    lab = [0] * 7
    # pick is an invalid row -> flagged without being visited
    cfg, flag, cnt = oracle.synthesize(x, [8, 4], valid, lab, [4], np.zeros(0, np.uint64), 0)
    assert list(flag) == [SYNTH] and cnt == 1
    np.testing.assert_array_equal(cfg, [[2, 1]])


def test_cluster_without_valid_member_is_dropped():
    x = np.array([[1, 1], [2, 2], [5, 5]], dtype=np.uint8)
    cfg, flag, cnt = oracle.synthesize(x, [8, 8], [0, 0, 1], [0, 0, 1], [0, 2], np.zeros(0, np.uint64), 0)
    assert list(flag) == [DROPPED, KEPT] and cnt == 1
    np.testing.assert_array_equal(cfg[0], [0, 0])


def test_replacement_equal_to_kept_pick_or_visited_is_dropped():
    # cluster 0: members (1,1),(1,1),(3,3); pick (3,3) visited; mode (1,1) equals cluster 1's kept pick
    x = np.array([[1, 1], [1, 1], [3, 3], [1, 1]], dtype=np.uint8)
    lab = [0, 0, 0, 1]
    cfg, flag, cnt = oracle.synthesize(x, [4, 4], None, lab, [2, 3], vis([3, 3]), 0)
    assert list(flag) == [DROPPED, KEPT] and cnt == 1
    # same, but the mode itself is visited
    x2 = np.array([[1, 1], [1, 1], [3, 3], [2, 2]], dtype=np.uint8)
    cfg, flag, cnt = oracle.synthesize(x2, [4, 4], None, lab, [2, 3], vis([3, 3], [1, 1]), 0)
    assert list(flag) == [DROPPED, KEPT] and cnt == 1


def test_two_flagged_clusters_with_equal_modes_second_dropped():
    # both clusters' picks are visited; both modes are (1,2): lower cluster keeps it
    x = np.array([[1, 2], [1, 2], [0, 2], [1, 2], [1, 2], [1, 3]], dtype=np.uint8)
    lab = [0, 0, 0, 1, 1, 1]
    cfg, flag, cnt = oracle.synthesize(x, [4, 4], None, lab, [2, 5], vis([0, 2], [1, 3]), 0)
    assert list(flag) == [SYNTH, DROPPED] and cnt == 1
    np.testing.assert_array_equal(cfg, [[1, 2], [0, 0]])


def test_empty_cluster_and_salted_membership():
    x = np.array([[1, 2], [3, 3]], dtype=np.uint8)
    # visited holds the hash of (1,2) under salt 9: a lookup with salt 0 must miss, with salt 9 hit
    v9 = vis([1, 2], salt=9)
    cfg, flag, cnt = oracle.synthesize(x, [4, 4], None, [0, 2], [0, -1, 1], v9, 0)
    assert list(flag) == [KEPT, EMPTY, KEPT] and cnt == 2
    cfg, flag, cnt = oracle.synthesize(x, [4, 4], None, [0, 2], [0, -1, 1], v9, 9)
    # flagged; its only member is itself -> mode (1,2) is visited -> dropped
    assert list(flag) == [DROPPED, EMPTY, KEPT] and cnt == 1


def test_adversarial_visited_flags_every_cluster():
    from paper_2001_08743_amd import workloads
    wl = workloads.random_task(77, n=400, d=5, n_blobs=6, ks=(6,), n_iter=10)
    x = wl.task_rows(0)
    sw = oracle.sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    lab, pick = oracle.snap(x, sw["centroids"][0, :6])
    visited = np.array(sorted({H(x[p], 0) for p in pick if p >= 0}), dtype=np.uint64)
    cfg, flag, cnt = oracle.synthesize(x, wl.cards[0], None, lab, pick, visited, 0)
    assert KEPT not in set(flag)
    for c in range(6):
        if flag[c] == SYNTH:
            members = x[lab == c]
            for j in range(x.shape[1]):
                counts = np.bincount(members[:, j], minlength=int(wl.cards[0, j]))
                assert cfg[c, j] == int(np.argmax(counts))      # argmax = first maximum = smallest value
            assert H(cfg[c], 0) not in set(int(v) for v in visited)


# ------------------------------------------------------------------ configuration updater

def test_updater_hand_worked_walk_with_clipping():
    theta = np.array([[0, 2], [3, 0]], dtype=np.uint8)
    cards = [4, 3]                                       # values 0..3 and 0..2
    actions = np.array([[[-1, +1], [+1, 0]],             # step 0: (0,2)->(0,2) both clipped; (3,0)->(3,0) clipped
                        [[+1, -1], [-1, +1]],            # step 1: (1,1); (2,1)
                        [[+1, 0], [0, 0]]], dtype=np.int8)   # step 2: (2,1) seen already; (2,1) again
    final, order = oracle.update_configs(theta, actions, cards)
    np.testing.assert_array_equal(final, [[2, 1], [2, 1]])
    assert order == [(0, 2), (3, 0), (1, 1), (2, 1)]


def test_updater_invariants():
    rng = np.random.default_rng(5)
    cards = rng.integers(1, 9, size=6)
    theta = (rng.random((10, 6)) * cards).astype(np.uint8)
    zero = np.zeros((4, 10, 6), dtype=np.int8)
    final, order = oracle.update_configs(theta, zero, cards)
    np.testing.assert_array_equal(final, theta)          # staying put changes nothing
    assert set(order) == set(map(tuple, theta.tolist()))
    up = np.ones((9, 10, 6), dtype=np.int8)              # enough steps up: everything ends at card - 1
    final, _ = oracle.update_configs(theta, up, cards)
    np.testing.assert_array_equal(final, np.broadcast_to(cards - 1, (10, 6)))
    final, _ = oracle.update_configs(theta, -up, cards)
    np.testing.assert_array_equal(final, np.zeros((10, 6)))
