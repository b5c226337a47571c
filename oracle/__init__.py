"""CPU oracle of the Adaptive Sampling hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes wrapper over ``cham_oracle.c`` (plain C, double precision; paper
Sec. 3.3 and Algorithm 1).  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; it imports nothing of the GPU
library and the GPU library imports nothing of it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cham_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

EMPTY, KEPT, SYNTH, DROPPED = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_hash.restype = C.c_uint64
        _lib.orc_hash.argtypes = [C.c_void_p, C.c_int, C.c_uint64]
        _lib.orc_select_k.restype = C.c_int
        _lib.orc_select_k.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double]
        _lib.orc_first_distinct.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _rows(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint16)
    assert x.ndim == 2
    return x


def num_threads() -> int:
    return int(lib().orc_num_threads())


def first_distinct(x, kmax: int) -> np.ndarray:
    x = _rows(x)
    out = np.zeros(kmax, dtype=np.int64)
    m = lib().orc_first_distinct(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), C.c_int(kmax), _p(out))
    return out[:m]


def kmeans(x, init_mu, n_iter: int, want_trace: bool = False):
    """Lloyd iteration for one k from the given start; returns dict(mu, counts, labels, inertia, trace)."""
    x = _rows(x)
    mu = np.array(init_mu, dtype=np.float64, order="C", copy=True)
    k, d = mu.shape
    assert d == x.shape[1]
    counts = np.zeros(k, dtype=np.int64)
    labels = np.zeros(x.shape[0], dtype=np.int32)
    inertia = np.zeros(1, dtype=np.float64)
    trace = np.zeros(n_iter + 1, dtype=np.float64) if want_trace else None
    lib().orc_kmeans(_p(x), C.c_int64(x.shape[0]), C.c_int(d), C.c_int(k), C.c_int(n_iter), _p(mu),
                     _p(counts), _p(labels), _p(inertia), _p(trace))
    return dict(mu=mu, counts=counts, labels=labels, inertia=float(inertia[0]), trace=trace)


def sweep(rows, task_off, ks: Sequence[int], n_iter: int, init: Optional[np.ndarray] = None,
          want_labels: bool = False, want_trace: bool = False):
    """Full sweep over ks for a batch of tasks; see ``orc_sweep`` for the layouts."""
    x = _rows(rows)
    task_off = np.ascontiguousarray(task_off, dtype=np.int64)
    T = len(task_off) - 1
    ks_a = np.ascontiguousarray(ks, dtype=np.int32)
    n_k = len(ks_a)
    d = x.shape[1]
    Ksum = int(ks_a.sum())
    n_total = int(task_off[-1])
    assert n_total == x.shape[0]
    cent = np.zeros((T, Ksum, d), dtype=np.float64)
    counts = np.zeros((T, Ksum), dtype=np.int64)
    inertia = np.zeros((T, n_k), dtype=np.float64)
    status = np.zeros((T, n_k), dtype=np.int32)
    labels = np.zeros((n_k, n_total), dtype=np.int32) if want_labels else None
    trace = np.zeros((T, n_k, n_iter + 1), dtype=np.float64) if want_trace else None
    init_a = None
    if init is not None:
        init_a = np.ascontiguousarray(init, dtype=np.float64)
        assert init_a.shape == cent.shape
    lib().orc_sweep(_p(x), C.c_int(d), _p(task_off), C.c_int(T), _p(ks_a), C.c_int(n_k),
                    C.c_int(n_iter), C.c_int(0 if init is None else 1), _p(init_a), _p(cent),
                    _p(counts), _p(inertia), _p(status), _p(labels), _p(trace))
    return dict(centroids=cent, counts=counts, inertia=inertia, status=status, labels=labels,
                trace=trace, koff=np.concatenate([[0], np.cumsum(ks_a)]).astype(np.int64))


def select_k(loss, status=None, threshold: float = 2.5) -> int:
    loss = np.ascontiguousarray(loss, dtype=np.float64)
    st = None if status is None else np.ascontiguousarray(status, dtype=np.int32)
    return int(lib().orc_select_k(_p(loss), _p(st), C.c_int(len(loss)), C.c_double(threshold)))


def sweep_until_knee(rows, task_off, ks: Sequence[int], n_iter: int, threshold: float = 2.5):
    """Algorithm 1's loop, one task at a time: for k in ks run k-means from the first k distinct rows;
    leave the loop at the first k with threshold * loss >= previous_loss (previous_loss starts at
    infinity); a k with fewer than k distinct rows is passed over.  Returns dict(chosen_idx [T],
    ran [T][n_k] bool, inertia [T][n_k], centroids: list per task of {ki: mu}, counts likewise)."""
    x = _rows(rows)
    task_off = np.ascontiguousarray(task_off, dtype=np.int64)
    T, n_k = len(task_off) - 1, len(ks)
    chosen = np.full(T, -1, dtype=np.int32)
    ran = np.zeros((T, n_k), dtype=bool)
    inertia = np.zeros((T, n_k), dtype=np.float64)
    cents, cnts = [], []
    for t in range(T):
        xt = x[task_off[t]:task_off[t + 1]]
        first = first_distinct(xt, int(max(ks))) if len(xt) else np.zeros(0, dtype=np.int64)
        previous_loss = np.inf
        last = -1
        cents.append({})
        cnts.append({})
        for ki, k in enumerate(ks):
            if len(first) < k:
                continue
            r = kmeans(xt, xt[first[:k]].astype(np.float64), n_iter)
            ran[t, ki] = True
            inertia[t, ki] = r["inertia"]
            cents[t][ki] = r["mu"]
            cnts[t][ki] = r["counts"]
            last = ki
            if threshold * r["inertia"] >= previous_loss:
                chosen[t] = ki
                break
            previous_loss = r["inertia"]
        if chosen[t] < 0:
            chosen[t] = last
    return dict(chosen_idx=chosen, ran=ran, inertia=inertia, centroids=cents, counts=cnts)


def update_configs(theta, actions, cards):
    """Configuration updater (Sec. 3.2): theta [B][d], actions [S][B][d] in {-1, 0, +1}, cards [d].
    Step after step theta <- clip(theta + a, 0, card - 1); returns (final theta, list of the distinct
    configurations reached, in order of first appearance: step by step, configuration by configuration)."""
    th = np.array(theta, dtype=np.int64, copy=True)
    acts = np.asarray(actions, dtype=np.int64)
    hi = np.asarray(cards, dtype=np.int64) - 1
    seen, order = set(), []
    for s in range(acts.shape[0]):
        for b in range(th.shape[0]):
            for j in range(th.shape[1]):
                v = th[b, j] + acts[s, b, j]
                if v < 0:
                    v = 0
                if v > hi[j]:
                    v = hi[j]
                th[b, j] = v
            key = tuple(int(v) for v in th[b])
            if key not in seen:
                seen.add(key)
                order.append(key)
    return th.astype(np.uint8), order


def snap(x, mu):
    x = _rows(x)
    mu = np.ascontiguousarray(mu, dtype=np.float64)
    k, d = mu.shape
    labels = np.zeros(x.shape[0], dtype=np.int32)
    pick = np.zeros(k, dtype=np.int64)
    lib().orc_snap(_p(x), C.c_int64(x.shape[0]), C.c_int(d), C.c_int(k), _p(mu), _p(labels), _p(pick))
    return labels, pick


def hash_config(cfg, salt: int = 0) -> int:
    cfg = np.ascontiguousarray(cfg, dtype=np.uint16)
    return int(lib().orc_hash(_p(cfg), C.c_int(cfg.shape[0]), C.c_uint64(int(salt))))


def hash_rows(x, salts) -> np.ndarray:
    """Hash every row; `salts` is one salt for all rows or one per row."""
    x = _rows(x)
    out = np.zeros(x.shape[0], dtype=np.uint64)
    if np.ndim(salts) == 0:
        lib().orc_hash_rows(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), None,
                            C.c_uint64(int(salts)), _p(out))
    else:
        s = np.ascontiguousarray(salts, dtype=np.uint64)
        assert len(s) == x.shape[0]
        lib().orc_hash_rows(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(s), C.c_uint64(0), _p(out))
    return out


def synthesize(x, cards, valid, labels, pick_row, visited_sorted, salt: int):
    x = _rows(x)
    d = x.shape[1]
    cards = np.ascontiguousarray(cards, dtype=np.uint16)
    assert cards.shape == (d,)
    if x.shape[0]:
        assert (x < cards[None, :]).all(), "knob value outside its cardinality"
    v = None if valid is None else np.ascontiguousarray(valid, dtype=np.uint8)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    pick_row = np.ascontiguousarray(pick_row, dtype=np.int64)
    k = len(pick_row)
    vis = np.ascontiguousarray(visited_sorted, dtype=np.uint64)
    assert (vis[1:] >= vis[:-1]).all()
    out_cfg = np.zeros((k, d), dtype=np.uint16)
    out_flag = np.zeros(k, dtype=np.uint8)
    out_count = np.zeros(1, dtype=np.int32)
    lib().orc_synthesize(_p(x), C.c_int64(x.shape[0]), C.c_int(d), _p(cards), _p(v), C.c_int(k),
                         _p(labels), _p(pick_row), _p(vis), C.c_int64(len(vis)), C.c_uint64(int(salt)),
                         _p(out_cfg), _p(out_flag), _p(out_count))
    return out_cfg, out_flag, int(out_count[0])


def visited_hashes(wl) -> np.ndarray:
    """Hashes (this oracle's hash) of the workload's visited configurations."""
    if len(wl.visited_cfg) == 0:
        return np.zeros(0, dtype=np.uint64)
    return hash_rows(wl.visited_cfg, wl.salts[wl.visited_task])


def pipeline(wl, visited_sorted, threshold: Optional[float] = None, sweep_out=None):
    """Sweep -> choose k -> snap -> synthesize for every task of a workload.

    Returns the sweep outputs plus, per task (k_max = max(ks)):
      chosen_idx [T], labels_sel [N_total], pick_row [T][k_max] (-1 beyond k* / empty),
      pick_cfg [T][k_max][d], out_cfg [T][k_max][d], out_flag [T][k_max], out_count [T].
    """
    thr = wl.threshold if threshold is None else threshold
    sw = sweep_out if sweep_out is not None else sweep(wl.rows, wl.task_off, wl.ks, wl.n_iter)
    T, d, kmax = wl.T, wl.d, max(wl.ks)
    chosen = np.full(T, -1, dtype=np.int32)
    labels_sel = np.zeros(wl.n_total, dtype=np.int32)
    pick_row = np.full((T, kmax), -1, dtype=np.int64)
    pick_cfg = np.zeros((T, kmax, d), dtype=np.uint16)
    out_cfg = np.zeros((T, kmax, d), dtype=np.uint16)
    out_flag = np.zeros((T, kmax), dtype=np.uint8)
    out_count = np.zeros(T, dtype=np.int32)
    for t in range(T):
        ci = select_k(sw["inertia"][t], sw["status"][t], thr)
        chosen[t] = ci
        if ci < 0:
            continue
        k = wl.ks[ci]
        x = wl.task_rows(t)
        mu = sw["centroids"][t, sw["koff"][ci]:sw["koff"][ci] + k]
        lab, pick = snap(x, mu)
        r0, r1 = wl.task_off[t], wl.task_off[t + 1]
        labels_sel[r0:r1] = lab
        pick_row[t, :k] = pick
        for c in range(k):
            if pick[c] >= 0:
                pick_cfg[t, c] = x[pick[c]]
        oc, of, cnt = synthesize(x, wl.cards[t], wl.task_valid(t), lab, pick, visited_sorted,
                                 int(wl.salts[t]))
        out_cfg[t, :k] = oc
        out_flag[t, :k] = of
        out_count[t] = cnt
    res = dict(sw)
    res.update(chosen_idx=chosen, labels_sel=labels_sel, pick_row=pick_row, pick_cfg=pick_cfg,
               out_cfg=out_cfg, out_flag=out_flag, out_count=out_count)
    return res
