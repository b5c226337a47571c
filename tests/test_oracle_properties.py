"""Property-based pins of the CPU oracle: on random small inputs every output is rebuilt from the
definition in plain Python (nearest centroid by exact rational distances, per-knob mode by
counting, membership by a Python set) and must agree.  Paper: Sec. 3.3 and Algorithm 1."""
from collections import Counter
from fractions import Fraction

import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from test_oracle_select_synth import H

KEPT, SYNTH, DROPPED, EMPTY = oracle.KEPT, oracle.SYNTH, oracle.DROPPED, oracle.EMPTY


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 5), st.integers(1, 6), st.integers(4, 40), st.integers(2, 700))
def test_one_lloyd_step_from_the_definition(seed, d, k, n, card):
    """Labels = exact nearest centroid (rational arithmetic, lowest index on ties); new centroids =
    means of the members; an empty cluster keeps its centroid; the loss is that of the final labels."""
    rng = np.random.default_rng(seed)
    x = rng.integers(0, card, size=(n, d)).astype(np.uint16)
    # centroids on a coarse rational grid: exactly representable in binary, so distances are exact in double
    mu = rng.integers(0, 4 * card, size=(k, d)) / 4.0
    r = oracle.kmeans(x, mu.copy(), 1)

    def label(row, cents):
        best, bi = None, -1
        for c in range(len(cents)):
            dist = sum((Fraction(int(row[j])) - Fraction(cents[c][j])) ** 2 for j in range(d))
            if best is None or dist < best:
                best, bi = dist, c
        return bi, best

    lab0 = [label(row, [[Fraction(v).limit_denominator(4) for v in m] for m in mu])[0] for row in x]
    new = []
    for c in range(k):
        members = [x[i] for i in range(n) if lab0[i] == c]
        if members:
            new.append([Fraction(sum(int(m[j]) for m in members), len(members)) for j in range(d)])
        else:
            new.append([Fraction(v).limit_denominator(4) for v in mu[c]])
    for c in range(k):
        for j in range(d):
            assert r["mu"][c, j] == float(new[c][j]) or abs(r["mu"][c, j] - float(new[c][j])) <= 1e-12 * max(1.0, abs(float(new[c][j])))
    # final labels: nearest of the new centroids as the oracle holds them (doubles), rows far from ties only
    cents = [[Fraction(float(r["mu"][c, j])) for j in range(d)] for c in range(k)]
    loss = Fraction(0)
    for i, row in enumerate(x):
        dists = sorted((sum((Fraction(int(row[j])) - cents[c][j]) ** 2 for j in range(d)), c) for c in range(k))
        if len(dists) == 1 or dists[1][0] - dists[0][0] > Fraction(1, 10 ** 6) * max(Fraction(1), dists[0][0]):
            assert r["labels"][i] == dists[0][1]
        loss += sum((Fraction(int(row[j])) - cents[r["labels"][i]][j]) ** 2 for j in range(d))
    assert abs(r["inertia"] - float(loss)) <= 1e-9 * max(1.0, float(loss))
    assert list(r["counts"]) == [int((r["labels"] == c).sum()) for c in range(k)]


@settings(max_examples=80, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 4), st.integers(1, 6), st.integers(3, 30), st.integers(2, 400),
       st.floats(0.0, 0.6), st.floats(0.0, 0.7))
def test_synthesis_from_the_definition(seed, d, k, n, card, p_invalid, p_visited):
    rng = np.random.default_rng(seed)
    cards = rng.integers(2, card + 1, size=d)
    x = np.stack([rng.integers(0, c, size=n) for c in cards], axis=1).astype(np.uint16)
    valid = (rng.random(n) >= p_invalid).astype(np.uint8)
    labels = rng.integers(0, k, size=n)
    pick = np.full(k, -1, dtype=np.int64)
    for c in range(k):
        members = np.where(labels == c)[0]
        if len(members):
            pick[c] = rng.choice(members)
    salt = int(rng.integers(0, 1000))
    visited_cfgs = [tuple(int(v) for v in x[i]) for i in range(n) if rng.random() < p_visited]
    visited_cfgs += [tuple(int(rng.integers(0, c)) for c in cards) for _ in range(3)]
    vis_set = {H(c, salt) for c in visited_cfgs}
    vis = np.array(sorted(vis_set), dtype=np.uint64)
    cfg, flag, cnt = oracle.synthesize(x, cards, valid, labels, pick, vis, salt)

    accepted = []          # configurations returned so far by lower clusters (SYNTH) plus all KEPT ones
    kept = {}
    for c in range(k):
        if pick[c] >= 0:
            row = tuple(int(v) for v in x[pick[c]])
            if valid[pick[c]] and H(row, salt) not in vis_set:
                kept[c] = row
    for c in range(k):
        if pick[c] < 0:
            assert flag[c] == EMPTY and not cfg[c].any()
            continue
        if c in kept:
            assert flag[c] == KEPT and tuple(int(v) for v in cfg[c]) == kept[c]
            continue
        members = [i for i in range(n) if labels[i] == c and valid[i]]
        want = None
        if members:
            mode = []
            for j in range(d):
                cntr = Counter(int(x[i, j]) for i in members)
                top = max(cntr.values())
                mode.append(min(v for v, q in cntr.items() if q == top))
            mode = tuple(mode)
            dup = H(mode, salt) in vis_set or mode in kept.values() or mode in accepted
            if not dup:
                want = mode
        if want is None:
            assert flag[c] == DROPPED and not cfg[c].any()
        else:
            assert flag[c] == SYNTH and tuple(int(v) for v in cfg[c]) == want
            accepted.append(want)
    assert cnt == len(kept) + len(accepted)


@settings(max_examples=80, deadline=None)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 4), st.integers(1, 5), st.integers(1, 25), st.integers(2, 300))
def test_snap_from_the_definition(seed, d, k, n, card):
    rng = np.random.default_rng(seed)
    x = rng.integers(0, card, size=(n, d)).astype(np.uint16)
    mu = rng.integers(0, 4 * card, size=(k, d)) / 4.0
    lab, pick = oracle.snap(x, mu)
    cents = [[Fraction(float(v)) for v in m] for m in mu]
    best = {}
    for i, row in enumerate(x):
        dists = [sum((Fraction(int(row[j])) - cents[c][j]) ** 2 for j in range(d)) for c in range(k)]
        c = min(range(k), key=lambda q: (dists[q], q))
        assert lab[i] == c
        if c not in best or dists[c] < best[c][0]:
            best[c] = (dists[c], i)
    for c in range(k):
        assert pick[c] == (best[c][1] if c in best else -1)
