"""Seeded synthetic tuning-task workloads (inputs only; no arithmetic of the method lives here).

The paper clusters candidate schedule configurations produced by its search
step (Sec. 3.3): each configuration is one integer choice per knob
(Sec. 2.2, Eq. 1; knob list in Table 1).  The paper's real candidates come
from tuning conv layers of AlexNet / VGG-16 / ResNet-18 inside a DNN
compiler, which is not available here, so these generators stand in for
them: integer knob-index vectors that form non-uniform clusters
(Sec. 3.3, "clustered in subregions ... non-uniformly distributed"),
a per-row validity mask (Sec. 3.3, invalid configurations) and a set of
already-measured configurations (Algorithm 1's visited set).

Both the CPU oracle's tests and the GPU binding's tests draw their inputs
from this module.  It deliberately knows nothing about distances, means,
modes or hashing: the visited set is handed out as *configurations* plus
raw random 64-bit words, and each side hashes them with its own hash.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

BASE_SEED = 20010874 * 10


@dataclass
class Workload:
    """One batch of independent tuning tasks.

    rows      u8  [N_total, d]   row-major knob-index vectors, tasks concatenated
    task_off  i64 [T+1]          rows of task t are [task_off[t], task_off[t+1])
    cards     u16 [T, d]         cardinality of knob j in task t (values are < card)
    valid     u8  [N_total]      1 = configuration is valid, 0 = known-invalid
    ks        list of int        the k values swept (strictly increasing)
    n_iter    int                Lloyd update steps per k
    threshold float              knee threshold (Table "threshold_meta" = 2.5)
    salts     u64 [T]            per-task hash salt (task id)
    visited_cfg  u8  [nv, d]     configurations already measured
    visited_task i64 [nv]        task each visited configuration belongs to
    visited_raw  u64 [nr]        random 64-bit words (stand for hashes of other configs)
    n_visited    int             target size of the visited set
    """

    name: str
    rows: np.ndarray
    task_off: np.ndarray
    cards: np.ndarray
    valid: np.ndarray
    ks: List[int]
    n_iter: int
    threshold: float
    salts: np.ndarray
    visited_cfg: np.ndarray
    visited_task: np.ndarray
    visited_raw: np.ndarray
    n_visited: int
    meta: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return len(self.task_off) - 1

    @property
    def d(self) -> int:
        return int(self.rows.shape[1])

    @property
    def n_total(self) -> int:
        return int(self.rows.shape[0])

    def task_rows(self, t: int) -> np.ndarray:
        return self.rows[self.task_off[t]:self.task_off[t + 1]]

    def task_valid(self, t: int) -> np.ndarray:
        return self.valid[self.task_off[t]:self.task_off[t + 1]]

    def nominal_evals(self) -> int:
        """Point-centroid distance evaluations of the full sweep: N * sum(k) * (n_iter + 1)."""
        return int(self.n_total) * int(sum(self.ks)) * (self.n_iter + 1)

    def subset(self, tasks: Sequence[int]) -> "Workload":
        """A workload holding only the listed tasks (same rows, same visited inputs)."""
        tasks = list(tasks)
        rows = np.concatenate([self.task_rows(t) for t in tasks], axis=0)
        valid = np.concatenate([self.task_valid(t) for t in tasks], axis=0)
        off = np.zeros(len(tasks) + 1, dtype=np.int64)
        off[1:] = np.cumsum([self.task_off[t + 1] - self.task_off[t] for t in tasks])
        remap = {t: i for i, t in enumerate(tasks)}
        keep = np.array([int(t) in remap for t in self.visited_task], dtype=bool)
        vt = np.array([remap[int(t)] for t in self.visited_task[keep]], dtype=np.int64)
        return Workload(
            name=f"{self.name}[tasks={tasks}]", rows=rows, task_off=off,
            cards=self.cards[tasks].copy(), valid=valid, ks=list(self.ks),
            n_iter=self.n_iter, threshold=self.threshold,
            salts=self.salts[tasks].copy(), visited_cfg=self.visited_cfg[keep].copy(),
            visited_task=vt, visited_raw=self.visited_raw.copy(),
            n_visited=self.n_visited, meta=dict(self.meta))


def conv_cards(rng: np.random.Generator) -> np.ndarray:
    """Cardinalities of the 12 split/unroll knobs of one conv2d template (Table 1).

    The eight named knobs give twelve index columns here: each 4-way split
    (tile_f, tile_y, tile_x) is carried as two index columns (outer and inner
    half of its factor tuple, 8..24 choices each), tile_rc as two columns and
    tile_ry, tile_rx as one column each (2-way splits, 4..8 choices), then
    auto_unroll_max_step (3 choices) and unroll_explicit (2 choices).
    Column order: f, y, x outer | rc, ry, rx | f, y, x inner | rc inner |
    auto_unroll | unroll_explicit.
    """
    c = np.empty(12, dtype=np.uint16)
    c[0:3] = rng.integers(8, 25, size=3)      # tile_f, tile_y, tile_x (outer index)
    c[3:6] = rng.integers(4, 9, size=3)       # tile_rc, tile_ry, tile_rx
    c[6:9] = rng.integers(8, 25, size=3)      # inner-split indices of tile_f/y/x
    c[9] = rng.integers(4, 9)                 # inner-split index of tile_rc
    c[10] = 3                                 # auto_unroll_max_step in {0, 512, 1500}
    c[11] = 2                                 # unroll_explicit in {0, 1}
    return c


def _blob_rows(rng, n, cards, n_blobs, sigma, dtype=np.uint8):
    """n integer rows from a non-uniform mixture of n_blobs Gaussian blobs in knob-index space.
    sigma is one number or one per knob."""
    d = len(cards)
    hi = cards.astype(np.float64) - 1.0
    centres = rng.random((n_blobs, d)) * hi
    weights = rng.dirichlet(np.ones(n_blobs))
    which = rng.choice(n_blobs, size=n, p=weights)
    pts = centres[which] + sigma * rng.standard_normal((n, d))
    pts = np.clip(np.rint(pts), 0.0, hi)
    return pts.astype(dtype)


def _spoil(rng, rows, valid, cards, frac):
    """Replace a fraction of rows by uniform-random knob vectors marked invalid."""
    n = rows.shape[0]
    m = int(round(frac * n))
    if m == 0:
        return
    idx = rng.choice(n, size=m, replace=False)
    for j, c in enumerate(cards):
        rows[idx, j] = rng.integers(0, int(c), size=m)
    valid[idx] = 0


def _visited(rng, rows_by_task, cards, n_visited, dtype=np.uint8):
    """Visited inputs: per task an equal share, half sampled from the task's rows (so that
    lookups hit), half uniform-random configurations; plus spare random words for topping up."""
    T = len(rows_by_task)
    d = rows_by_task[0].shape[1]
    if n_visited <= 0:
        return (np.zeros((0, d), dtype), np.zeros(0, np.int64), np.zeros(0, np.uint64))
    per = max(2, n_visited // T)
    cfgs, tasks = [], []
    for t in range(T):
        r = rows_by_task[t]
        h = per // 2
        pick = rng.choice(r.shape[0], size=min(h, r.shape[0]), replace=False)
        cfgs.append(r[pick])
        rnd = np.stack([rng.integers(0, int(c), size=per - h) for c in cards[t]], axis=1)
        cfgs.append(rnd.astype(dtype))
        tasks.append(np.full(len(pick) + (per - h), t, dtype=np.int64))
    cfg = np.concatenate(cfgs, axis=0)
    task = np.concatenate(tasks, axis=0)
    raw = rng.integers(0, 2 ** 63, size=n_visited + 1024, dtype=np.uint64) * np.uint64(2) \
        + rng.integers(0, 2, size=n_visited + 1024, dtype=np.uint64)
    return cfg, task, raw


def finalize_visited(hashes: np.ndarray, raw: np.ndarray, size: int) -> np.ndarray:
    """Sorted, duplicate-free visited array of exactly `size` words: the given hashes of the
    visited configurations (computed by the caller with its own hash), topped up from `raw`."""
    have = np.unique(np.asarray(hashes, dtype=np.uint64))
    if size <= 0:
        return np.zeros(0, dtype=np.uint64)
    if len(have) > size:
        return have[:size].copy()
    i = 0
    raw = np.asarray(raw, dtype=np.uint64)
    while len(have) < size:
        need = size - len(have)
        if i + need > len(raw):
            raise ValueError("not enough spare words to fill the visited set")
        have = np.unique(np.concatenate([have, raw[i:i + need]]))
        i += need
    return have


def _assemble(name, rng, task_sizes, card_list, blobs, sigma, invalid_frac, ks, n_iter,
              n_visited, threshold=2.5, meta=None, dtype=np.uint8, sigma_rel=0.0):
    """sigma_rel > 0: the spread of knob j is max(sigma, sigma_rel * card_j) index steps."""
    rows_by_task, valid_by_task = [], []
    for n, cards, b in zip(task_sizes, card_list, blobs):
        sg = np.maximum(sigma, sigma_rel * cards.astype(np.float64)) if sigma_rel > 0 else sigma
        r = _blob_rows(rng, n, cards, b, sg, dtype)
        v = np.ones(n, dtype=np.uint8)
        _spoil(rng, r, v, cards, invalid_frac)
        rows_by_task.append(r)
        valid_by_task.append(v)
    cards = np.stack(card_list).astype(np.uint16)
    vcfg, vtask, vraw = _visited(rng, rows_by_task, cards, n_visited, dtype)
    off = np.zeros(len(task_sizes) + 1, dtype=np.int64)
    off[1:] = np.cumsum(task_sizes)
    T = len(task_sizes)
    m = dict(meta or {})
    m.update(blobs=[int(b) for b in blobs], sigma=float(sigma), invalid_frac=float(invalid_frac))
    return Workload(name=name, rows=np.ascontiguousarray(np.concatenate(rows_by_task, axis=0)),
                    task_off=off, cards=cards, valid=np.concatenate(valid_by_task),
                    ks=list(ks), n_iter=int(n_iter), threshold=float(threshold),
                    salts=np.arange(T, dtype=np.uint64), visited_cfg=vcfg, visited_task=vtask,
                    visited_raw=vraw, n_visited=int(n_visited), meta=m)


def make_config(cfg: int, seed_index: int = 0, scale: float = 1.0) -> Workload:
    """Workload number `cfg` (1..5) of the benchmark list; `seed_index` selects extra seeds.

    `scale` < 1 shrinks the number of tasks (configs 3, 5) or rows (config 4) for quick tests;
    the bench and the full-size parity tests use scale = 1.
    """
    rng = np.random.default_rng(BASE_SEED + cfg + 1000 * seed_index)
    if cfg == 1:     # tiny single task
        cards = rng.integers(2, 17, size=8).astype(np.uint16)
        return _assemble("cfg1-tiny", rng, [256], [cards], [6], 1.0, 0.0,
                         range(2, 17), 30, 0)
    if cfg == 2:     # one conv2d-layer design space
        cards = conv_cards(rng)
        return _assemble("cfg2-conv2d", rng, [4096], [cards], [16], 1.5, 0.05,
                         range(2, 65), 50, 4096)
    if cfg == 3:     # batched tuning tasks
        T = max(1, int(round(64 * scale)))
        card_list = [conv_cards(rng) for _ in range(T)]
        blobs = rng.integers(8, 25, size=T)
        return _assemble("cfg3-batched", rng, [1024] * T, card_list, blobs, 1.5, 0.05,
                         range(2, 33), 30, 65536 if scale == 1.0 else max(64, int(65536 * scale)))
    if cfg == 4:     # one large clustering
        n = max(1024, int(round(1048576 * scale)))
        cards = rng.integers(2, 33, size=16).astype(np.uint16)
        return _assemble("cfg4-large", rng, [n], [cards], [128], 2.0, 0.0,
                         [16, 32, 64, 128, 256], 20, 0)
    if cfg == 5:     # full-model sweep
        T = max(1, int(round(256 * scale)))
        card_list = [rng.integers(2, 33, size=24).astype(np.uint16) for _ in range(T)]
        blobs = rng.integers(4, 65, size=T)
        return _assemble("cfg5-fullmodel", rng, [4096] * T, card_list, blobs, 1.5, 0.05,
                         range(1, 65), 50, 1048576 if scale == 1.0 else max(64, int(1048576 * scale)))
    raise ValueError("cfg must be 1..5")


def random_task(seed: int, n: int, d: int, card_lo: int = 2, card_hi: int = 16, n_blobs: int = 4,
                sigma: float = 1.0, invalid_frac: float = 0.0, ks=(2, 3, 4), n_iter: int = 10,
                n_visited: int = 0, n_tasks: int = 1, ragged: bool = False) -> Workload:
    """Small free-form workload for unit and edge-case tests."""
    rng = np.random.default_rng(seed)
    sizes = [n] * n_tasks
    if ragged:
        sizes = [max(1, int(n * f)) for f in rng.uniform(0.3, 1.0, size=n_tasks)]
    card_list = [rng.integers(card_lo, card_hi + 1, size=d).astype(np.uint16) for _ in range(n_tasks)]
    return _assemble(f"rand-{seed}", rng, sizes, card_list, [n_blobs] * n_tasks, sigma,
                     invalid_frac, ks, n_iter, n_visited)


def wide_space(seed: int, n_tasks: int = 64, n: int = 2048, d: int = 40, ks=range(2, 33), n_iter: int = 30,
               n_visited: int = 4096, wide_frac: float = 0.3, card_wide=(64, 600), card_small=(2, 32),
               ragged: bool = False) -> Workload:
    """Tuning tasks over design spaces with two-byte knobs (Sec. 2: the product of the knobs' choice
    lists reaches 10^10 points; a split knob of a large loop has hundreds of choices): a share
    `wide_frac` of the knobs draws its cardinality from `card_wide`, the others from `card_small`;
    8..24 blobs per task whose spread is max(1.5, 2 % of the cardinality) index steps per knob;
    5 % uniform-random invalid rows.  Rows are uint16."""
    rng = np.random.default_rng(BASE_SEED * 7 + seed)
    sizes = [n] * n_tasks
    if ragged:
        sizes = [max(1, int(n * f)) for f in rng.uniform(0.3, 1.0, size=n_tasks)]
    card_list = []
    for _ in range(n_tasks):
        wide = rng.random(d) < wide_frac
        c = np.where(wide, rng.integers(card_wide[0], card_wide[1] + 1, size=d),
                     rng.integers(card_small[0], card_small[1] + 1, size=d))
        card_list.append(c.astype(np.uint16))
    blobs = rng.integers(8, 25, size=n_tasks)
    return _assemble(f"wide-{seed}", rng, sizes, card_list, blobs, 1.5, 0.05, ks, n_iter, n_visited,
                     dtype=np.uint16, sigma_rel=0.02)


def random_workload(seed: int) -> Workload:
    """A small workload of random shape for randomised parity tests: 1..5 ragged tasks (a quarter of
    the draws with tasks of up to 9000 rows, else up to 2500), byte knobs (d = 1..31, cardinalities up
    to 4 / 16 / 64 / 256) or, for a third of the draws, two-byte knobs (d = 1..64, two fifths of
    the knobs with cardinalities up to 300 / 2048 / 5000), 1..6 values of k up to 3..256, 0..14 Lloyd
    steps, 1..19 blobs per task of spread 0.5 / 1.5 / 3, 5 % invalid rows."""
    rng = np.random.default_rng(BASE_SEED * 11 + seed)
    wide = rng.random() < 0.35
    d = int(rng.integers(1, 65 if wide else 32))
    T = int(rng.integers(1, 6))
    big = rng.random() < 0.25
    sizes = [int(rng.integers(1, 9000 if big else 2500)) for _ in range(T)]
    kmax = int(rng.choice([3, 8, 16, 31, 32, 33, 64, 100, 256]))
    if wide:
        kmax = min(kmax, 100 if d <= 48 else 64)
    ks = sorted(set(int(x) for x in rng.integers(1, kmax + 1, size=int(rng.integers(1, 6)))) | {kmax})
    n_iter = int(rng.choice([0, 1, 2, 5, 9, 14]))
    if wide:
        hi = int(rng.choice([300, 2048, 5000]))
        card_list = [np.where(rng.random(d) < 0.4, rng.integers(2, hi + 1, size=d),
                              rng.integers(2, 33, size=d)).astype(np.uint16) for _ in range(T)]
    else:
        hi = int(rng.choice([4, 16, 64, 256]))
        card_list = [rng.integers(1 if d == 1 else 2, hi + 1, size=d).astype(np.uint16) for _ in range(T)]
    blobs = rng.integers(1, 20, size=T)
    sigma = float(rng.choice([0.5, 1.5, 3.0]))
    return _assemble(f"random-{seed}", rng, sizes, card_list, blobs, sigma, 0.05, ks, n_iter,
                     int(rng.integers(1, 400)), threshold=float(rng.choice([1.05, 1.3, 2.5])),
                     dtype=np.uint16 if wide else np.uint8, sigma_rel=0.02 if wide else 0.0)
