"""Seeded generators for Criteo-shaped embedding workloads.

The paper trains on Criteo Kaggle and Criteo Terabyte (its experiments
section; model shapes in its model-architecture table: 26 tables, at most
about 10 M rows per table, embedding width 16 or 64).  Neither dataset is
available here, so these generators stand in for them: same table count, same
widths, a comparable spread of table sizes (3 rows up to 10 M rows), totals
chosen so that the fp32 model sizes match the paper's 2.16 GB / 12.58 GB, and
power-law (Zipf) row popularity as in click logs.

Everything is a pure function of (config, seed, batch number); all draws use
``numpy.random.Generator(PCG64(SeedSequence([...])))`` so that any piece can be
regenerated independently and in parallel.  No quantisation, pooling,
deduplication or update arithmetic lives here.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

# name -> shape of the workload.  ``rows`` is the total over tables.
CONFIGS: Dict[str, dict] = {
    # 4 tables x 1000 rows x dim 16, batch 128, uniform indices
    "tiny": dict(T=4, D=16, B=128, alpha=None, rows=4000, fixed_card=1000, seed=1001),
    # 1 table, 1 M rows x dim 16, batch 2048, Zipf 1.05
    "single": dict(T=1, D=16, B=2048, alpha=1.05, rows=1_000_000, fixed_card=1_000_000, seed=1002),
    # Kaggle-shaped: 26 tables, ~33.77 M rows (2.161 GB fp32), dim 16, batch 2048
    "kaggle": dict(T=26, D=16, B=2048, alpha=1.05, rows=33_770_000, fixed_card=None, seed=1003),
    # Terabyte-shaped: 26 tables, ~49.12 M rows (12.575 GB fp32), dim 64, batch 8192
    "terabyte": dict(T=26, D=64, B=8192, alpha=1.1, rows=49_120_000, fixed_card=None, seed=1004),
}

CARD_MIN = 3
CARD_MAX = 10_000_000

_STREAM_CARDS, _STREAM_TABLE, _STREAM_MAP, _STREAM_BATCH, _STREAM_GRAD = 1, 2, 3, 4, 5


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def cardinalities(T: int, total_rows: int, seed: int) -> np.ndarray:
    """Table sizes: log-uniform in [3, 1e7], rescaled to ``total_rows`` with a cap.

    Tables that hit the cap stay there; the others are scaled by a common
    factor until the total matches, then rounded, and the rounding residue is
    absorbed by the largest uncapped table.
    """
    rng = _rng(seed, _STREAM_CARDS)
    c = np.exp(rng.uniform(math.log(CARD_MIN), math.log(CARD_MAX), size=T))
    for _ in range(64):
        c = np.clip(c, CARD_MIN, CARD_MAX)
        free = c < CARD_MAX
        need = total_rows - c[~free].sum()
        have = c[free].sum()
        if have <= 0 or abs(c.sum() - total_rows) < 0.5:
            break
        c[free] *= need / have
    cards = np.clip(np.rint(c), CARD_MIN, CARD_MAX).astype(np.int64)
    free_idx = np.flatnonzero(cards < CARD_MAX)
    if free_idx.size:
        j = free_idx[np.argmax(cards[free_idx])]
        cards[j] = min(CARD_MAX, max(CARD_MIN, cards[j] + (total_rows - int(cards.sum()))))
    return cards


def _fill_table(out: np.ndarray, rows: int, seed: int, t: int, chunk_rows: int = 1 << 18) -> None:
    """U(-1/sqrt(rows), +1/sqrt(rows)) in fp32, written in place (the paper
    says tables start from a uniform initialisation; the bound is the usual
    embedding-table one)."""
    rng = _rng(seed, _STREAM_TABLE, t)
    bound = np.float32(1.0 / math.sqrt(rows))
    D = out.shape[1]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        u = rng.random((r1 - r0, D), dtype=np.float32)
        np.multiply(u, np.float32(2.0), out=u)
        np.subtract(u, np.float32(1.0), out=u)
        np.multiply(u, bound, out=out[r0:r1])


def make_tables(cards: np.ndarray, D: int, seed: int, threads: int = 8,
                out: Optional[np.ndarray] = None) -> np.ndarray:
    """All tables concatenated, [sum(cards), D] fp32, row-major."""
    R = int(cards.sum())
    if out is None:
        out = np.empty((R, D), dtype=np.float32)
    offs = np.concatenate([[0], np.cumsum(cards)])
    jobs = [(out[offs[t]:offs[t + 1]], int(cards[t]), seed, t) for t in range(len(cards))]
    if threads <= 1:
        for j in jobs:
            _fill_table(*j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda j: _fill_table(*j), jobs))
    return out


def _coprime_multiplier(rows: int, rng: np.random.Generator) -> int:
    if rows <= 2:
        return 1
    a = int(rng.integers(1, rows))
    while math.gcd(a, rows) != 1:
        a += 1
        if a >= rows:
            a = 1
    return a


@dataclass
class Workload:
    name: str
    T: int
    D: int
    B: int
    alpha: Optional[float]
    seed: int
    cards: np.ndarray
    row_offsets: np.ndarray = field(init=False)
    _cdf: dict = field(default_factory=dict, repr=False)
    _map: dict = field(default_factory=dict, repr=False)

    def __post_init__(self) -> None:
        self.cards = np.asarray(self.cards, dtype=np.int64)
        self.row_offsets = np.concatenate([[0], np.cumsum(self.cards)]).astype(np.int64)

    @property
    def R(self) -> int:
        return int(self.row_offsets[-1])

    def tables(self, threads: int = 8) -> np.ndarray:
        return make_tables(self.cards, self.D, self.seed, threads=threads)

    # ---- index batches -------------------------------------------------
    def _zipf_cdf(self, t: int) -> np.ndarray:
        cdf = self._cdf.get(t)
        if cdf is None:
            rows = int(self.cards[t])
            w = np.arange(1, rows + 1, dtype=np.float64) ** (-float(self.alpha))
            cdf = np.cumsum(w)
            cdf /= cdf[-1]
            self._cdf[t] = cdf
        return cdf

    def _rank_to_row(self, t: int) -> Tuple[int, int]:
        ab = self._map.get(t)
        if ab is None:
            rows = int(self.cards[t])
            rng = _rng(self.seed, _STREAM_MAP, t)
            a = _coprime_multiplier(rows, rng)
            b = int(rng.integers(0, rows))
            ab = (a, b)
            self._map[t] = ab
        return ab

    def _draw_rows(self, t: int, n: int, rng: np.random.Generator) -> np.ndarray:
        rows = int(self.cards[t])
        if self.alpha is None:
            return rng.integers(0, rows, size=n, dtype=np.int64)
        cdf = self._zipf_cdf(t)
        k = np.searchsorted(cdf, rng.random(n), side="right")
        k = np.minimum(k, rows - 1).astype(np.int64)  # rank-1 in [0, rows)
        a, b = self._rank_to_row(t)
        return (a * k + b) % rows

    def batch(self, k: int, pooling: str = "one", max_len: int = 4) -> Tuple[np.ndarray, np.ndarray]:
        """Batch number ``k``: ``(indices [N] int64 table-major, offsets [T*B+1] int64)``.

        ``pooling="one"``: exactly one index per bag (all of the paper-shaped
        configs).  ``pooling="ragged"``: bag lengths uniform in [0, max_len],
        so empty bags and uneven bags occur.  ``pooling="fixed"``: every bag has
        ``max_len`` indices (a pooling factor).
        """
        rng = _rng(self.seed, _STREAM_BATCH, k)
        T, B = self.T, self.B
        if pooling == "one":
            lens = np.ones(T * B, dtype=np.int64)
        elif pooling == "ragged":
            lens = rng.integers(0, max_len + 1, size=T * B, dtype=np.int64)
        elif pooling == "fixed":
            lens = np.full(T * B, max_len, dtype=np.int64)
        else:
            raise ValueError(pooling)
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        parts = []
        for t in range(T):
            n_t = int(offsets[(t + 1) * B] - offsets[t * B])
            parts.append(self._draw_rows(t, n_t, rng))
        indices = np.concatenate(parts) if parts else np.empty(0, np.int64)
        return np.ascontiguousarray(indices, dtype=np.int64), offsets

    # ---- upstream gradients -------------------------------------------
    def grad_dyadic(self, k: int) -> np.ndarray:
        return grad_dyadic(self.B, self.T, self.D, self.seed, k)

    def grad_normal(self, k: int) -> np.ndarray:
        return grad_normal(self.B, self.T, self.D, self.seed, k)


def make_workload(name: str, **override) -> Workload:
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    T = cfg["T"]
    if cfg.get("fixed_card"):
        cards = np.full(T, cfg["fixed_card"], dtype=np.int64)
    else:
        cards = cardinalities(T, cfg["rows"], cfg["seed"])
    return Workload(name=name, T=T, D=cfg["D"], B=cfg["B"], alpha=cfg["alpha"], seed=cfg["seed"], cards=cards)


def index_batch(wl: Workload, k: int, **kw):
    return wl.batch(k, **kw)


def split_batch(indices: np.ndarray, offsets: np.ndarray, T: int, B: int, parts: int):
    """Cuts a batch of B samples into ``parts`` micro-batches of B / parts consecutive samples (the split of
    the batch over simulated nodes): a list of ``(indices_k, offsets_k)`` in the same table-major layout."""
    assert B % parts == 0
    Bm = B // parts
    out = []
    for k in range(parts):
        idx, lens = [], []
        for t in range(T):
            lo, hi = int(offsets[t * B + k * Bm]), int(offsets[t * B + (k + 1) * Bm])
            idx.append(indices[lo:hi])
            lens.append(np.diff(offsets[t * B + k * Bm: t * B + (k + 1) * Bm + 1]))
        off = np.concatenate([[0], np.cumsum(np.concatenate(lens))]).astype(np.int64)
        out.append((np.ascontiguousarray(np.concatenate(idx), dtype=np.int64), off))
    return out


def grad_dyadic(B: int, T: int, D: int, seed: int, k: int) -> np.ndarray:
    """Gradient w.r.t. the pooled output, [B, T, D] fp32, on the grid m * 2^-24
    with integer m uniform in [-1024, 1024].  Any sum of at most 8192 such
    values is exactly representable in fp32, so every summation order gives
    the same bits and the sum has an integer closed form."""
    rng = _rng(seed, _STREAM_GRAD, 0, k)
    m = rng.integers(-1024, 1025, size=(B, T, D), dtype=np.int32)
    return (m.astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def grad_normal(B: int, T: int, D: int, seed: int, k: int) -> np.ndarray:
    """Gradient w.r.t. the pooled output, [B, T, D] fp32, N(0, 1e-4^2)."""
    rng = _rng(seed, _STREAM_GRAD, 1, k)
    g = rng.standard_normal(size=(B, T, D), dtype=np.float32)
    g *= np.float32(1e-4)
    return g


# ---- the dense part of the model (the "full train step" configuration) ---------------
DENSE_CONFIGS = {
    # Kaggle shape: 13 dense features, bottom MLP 13-512-256-64-16, top MLP 367-512-256-1
    "kaggle": dict(num_dense=13, bot=[13, 512, 256, 64, 16], top_hidden=[512, 256, 1]),
    # a small shape with the same structure and awkward (non-multiple-of-tile) widths
    "small": dict(num_dense=5, bot=[5, 40, 16], top_hidden=[70, 33, 1]),
    "small8": dict(num_dense=5, bot=[5, 24, 8], top_hidden=[19, 7, 1]),
    # mid-size, awkward widths: reductions of a few slabs with ragged ends, tiles that end past the edge
    "medium": dict(num_dense=7, bot=[7, 200, 96, 24], top_hidden=[136, 72, 1]),
    # a bottom MLP of a single layer; a first layer whose width is not a multiple of 4; one with a longer input
    "one_layer": dict(num_dense=9, bot=[9, 16], top_hidden=[33, 1]),
    "odd_first": dict(num_dense=6, bot=[6, 30, 16], top_hidden=[21, 1]),
    "long_first": dict(num_dense=20, bot=[20, 44, 16], top_hidden=[40, 12, 1]),
}

_STREAM_DENSE = 6


def make_dense_model(name: str, T: int, D: int, seed: int):
    """Seeded parameters of the MLPs: W_l ~ N(0, 2/(in+out)) and b_l ~ N(0, 1/out) in fp32 (the usual DLRM
    initialisation; the paper gives only the layer widths).  Returns (bot_dims, bot_w, bot_b, top_dims, top_w,
    top_b) with W_l of shape [out][in]."""
    cfg = DENSE_CONFIGS[name]
    bot_dims = list(cfg["bot"])
    assert bot_dims[-1] == D
    V = T + 1
    top_dims = [D + V * (V - 1) // 2] + list(cfg["top_hidden"])
    rng = _rng(seed, _STREAM_DENSE, 0)

    def layers(dims):
        ws, bs = [], []
        for i, o in zip(dims[:-1], dims[1:]):
            ws.append((rng.standard_normal((o, i)) * math.sqrt(2.0 / (i + o))).astype(np.float32))
            bs.append((rng.standard_normal(o) * math.sqrt(1.0 / o)).astype(np.float32))
        return ws, bs

    bw, bb = layers(bot_dims)
    tw, tb = layers(top_dims)
    return bot_dims, bw, bb, top_dims, tw, tb


def dense_batch(B: int, num_dense: int, seed: int, k: int):
    """Dense features exp(N(0,1)) [B][num_dense] fp32 and labels Bernoulli(0.25) [B] fp32."""
    rng = _rng(seed, _STREAM_DENSE, 1, k)
    x = np.exp(rng.standard_normal((B, num_dense))).astype(np.float32)
    y = (rng.random(B) < 0.25).astype(np.float32)
    return x, y
