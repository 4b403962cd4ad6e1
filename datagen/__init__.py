"""Seeded synthetic inputs for the factorized-learning hot path.

This module only draws random tables, index arrays and column maps in the shapes the
benchmark configurations name.  It contains none of the method's arithmetic: no join, no
matrix product, no gradient.  Labels that depend on ``T @ w*`` are finished by
:func:`finish_labels`, which receives that product from whichever side (the CPU oracle in
the tests, the device library in the benchmark) computed it.

Both the CPU oracle's tests and the device path's tests draw from here so that they see
the same bits.

Representation (notation of the paper's Sec. 2.1):

* ``Source.D``       -- source table ``D_k`` (``S_k`` in the paper), ``r_k x c_k`` float32, row-major.
* ``Source.row_idx`` -- compressed indicator matrix ``I_k`` (Def. 2): ``int32[r_T]``, entry ``i`` is
  the row of ``D_k`` that feeds target row ``i`` or ``-1``; ``None`` means the identity.
* ``Source.col_map`` -- compressed mapping matrix ``M_k`` (Def. 1): ``int32[c_k]``, entry ``j`` is the
  target column of source column ``j`` or ``-1``.

Every generator documents its draw order; all randomness comes from
``numpy.random.Generator(PCG64(seed))``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

__all__ = [
    "Source", "Schema", "rng_for", "star_schema", "config0", "config1", "config2", "config3",
    "config4", "tiny_random_schema", "bounded_zipf_keys", "finish_labels", "CONFIG1_GRID", "sparsify",
    "OneHotTable", "one_hot_star", "MOVIE_SHAPE",
]


@dataclass
class Source:
    D: np.ndarray                       # float32 [r_k, c_k]
    row_idx: Optional[np.ndarray]       # int32 [r_T] or None (identity)
    col_map: np.ndarray                 # int32 [c_k]

    @property
    def rows(self) -> int:
        return int(self.D.shape[0])

    @property
    def cols(self) -> int:
        return int(self.D.shape[1])


@dataclass
class Schema:
    sources: List[Source]
    r_T: int
    c_T: int
    extras: Dict[str, np.ndarray] = field(default_factory=dict)   # w_star, noise, X, Y, lr ...
    name: str = ""


def rng_for(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _normal32(rng: np.random.Generator, shape) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    # A signed zero would make "select" and "0 + x" differ in the last bit pattern.
    out[out == 0.0] = 0.0
    return out


def bounded_zipf_keys(rng: np.random.Generator, n_draws: int, n_keys: int, s: float) -> np.ndarray:
    """Keys in [0, n_keys) whose popularity follows a bounded Zipf law with exponent ``s``.

    Draw order: ``n_draws`` uniforms (inverse-CDF over ranks 1..n_keys), then one permutation of
    the keys that decides which key holds which rank.
    """
    ranks = np.arange(1, n_keys + 1, dtype=np.float64)
    pmf = ranks ** (-s)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    u = rng.random(n_draws)
    rank0 = np.searchsorted(cdf, u, side="left")
    rank0 = np.minimum(rank0, n_keys - 1)
    rank_to_key = rng.permutation(n_keys)
    return rank_to_key[rank0].astype(np.int32)


def star_schema(rng: np.random.Generator, r_S: int, c_S: int, dims, name: str = "") -> Schema:
    """Entity table ``S`` plus dimension tables joined through foreign keys.

    ``dims`` is a list of ``(rows, cols, fk_kind)`` with ``fk_kind`` in ``{"uniform", ("zipf", s)}``.
    Target columns are the disjoint blocks ``[S | R_1 | R_2 | ...]``.
    Draw order: S, then for each dimension its table followed by its foreign keys.
    """
    c_T = c_S + sum(d[1] for d in dims)
    sources = [Source(_normal32(rng, (r_S, c_S)), None, np.arange(c_S, dtype=np.int32))]
    off = c_S
    for rows, cols, kind in dims:
        R = _normal32(rng, (rows, cols))
        if kind == "uniform":
            fk = rng.integers(0, rows, size=r_S, dtype=np.int32)
        else:
            fk = bounded_zipf_keys(rng, r_S, rows, float(kind[1]))
        sources.append(Source(R, fk, np.arange(off, off + cols, dtype=np.int32)))
        off += cols
    return Schema(sources, r_S, c_T, name=name)


def config0(seed: int = 0, r_S: int = 10_000, r_R: int = 1_000) -> Schema:
    """Two-source star join for linear regression: S r_S x 4, R r_R x 8, uniform keys.

    Draw order: S, R, fk, w_star (12), noise (r_S, sigma 0.01).
    """
    rng = rng_for(seed)
    sch = star_schema(rng, r_S, 4, [(r_R, 8, "uniform")], name="config0")
    sch.extras["w_star"] = rng.standard_normal(sch.c_T)
    sch.extras["noise"] = 0.01 * rng.standard_normal(r_S)
    sch.extras["lr"] = np.array([0.1])
    sch.extras["iters"] = np.array([20])
    return sch


CONFIG1_GRID = [(r, c) for r in (10_000, 100_000, 500_000) for c in (20, 200, 800)]


def config1(seed: int = 1, r_S: int = 1_000_000, c_S: int = 20, r_R: int = 100_000,
            c_R: int = 200) -> Schema:
    """Operator micro-benchmark star join.  Draw order: S, R, fk, X1, X16, Y1, Y16."""
    rng = rng_for(seed)
    sch = star_schema(rng, r_S, c_S, [(r_R, c_R, "uniform")], name=f"config1[{r_R}x{c_R}]")
    sch.extras["X1"] = _normal32(rng, (sch.c_T, 1))
    sch.extras["X16"] = _normal32(rng, (sch.c_T, 16))
    sch.extras["Y1"] = _normal32(rng, (r_S, 1))
    sch.extras["Y16"] = _normal32(rng, (r_S, 16))
    return sch


def config2(seed: int = 2, r_S: int = 5_000_000, dim_rows=(100_000, 50_000, 10_000)) -> Schema:
    """Three-dimension star schema for logistic regression; the second key is Zipf(1.1).

    Draw order: S, R1, fk1, R2, fk2 (uniforms then rank permutation), R3, fk3, w_star
    (variance 1/200), noise (sigma 0.1).
    """
    rng = rng_for(seed)
    dims = [(dim_rows[0], 50, "uniform"), (dim_rows[1], 100, ("zipf", 1.1)),
            (dim_rows[2], 40, "uniform")]
    sch = star_schema(rng, r_S, 10, dims, name="config2")
    sch.extras["w_star"] = rng.standard_normal(sch.c_T) / np.sqrt(200.0)
    sch.extras["noise"] = 0.1 * rng.standard_normal(r_S)
    sch.extras["lr"] = np.array([0.5])
    sch.extras["iters"] = np.array([50])
    return sch


def config3(seed: int = 3, rows: int = 2_000_000, cols: int = 64, shared: int = 32,
            overlap: float = 0.3) -> Schema:
    """Union-style integration of two sources that share ``shared`` columns and some entities.

    Target rows are all rows of S1 followed by the rows of S2 that match no S1 row, in S2 order.
    Target columns are ``[S1-only | shared | S2-only]``.  A matched S2 row lands on the target row of
    its S1 partner; its copies of the shared cells are zeroed in ``D_2`` so that the cell comes from
    S1 alone.  Draw order: S1, S2, permutation of S2 rows (first ``n_match`` are the matched ones),
    permutation of S1 rows (first ``n_match`` are their partners), w_star, noise (sigma 0.01).
    """
    rng = rng_for(seed)
    S1 = _normal32(rng, (rows, cols))
    S2 = _normal32(rng, (rows, cols))
    n_match = int(round(overlap * rows))
    matched_s2 = rng.permutation(rows)[:n_match]
    partner_s1 = rng.permutation(rows)[:n_match]
    is_matched = np.zeros(rows, dtype=bool)
    is_matched[matched_s2] = True
    new_s2 = np.flatnonzero(~is_matched)
    r_T = rows + new_s2.size
    c_T = 2 * cols - shared
    idx1 = np.full(r_T, -1, dtype=np.int32)
    idx1[:rows] = np.arange(rows, dtype=np.int32)
    idx2 = np.full(r_T, -1, dtype=np.int32)
    idx2[partner_s1] = matched_s2.astype(np.int32)
    idx2[rows:] = new_s2.astype(np.int32)
    S2[matched_s2, :shared] = 0.0
    cm1 = np.arange(cols, dtype=np.int32)
    cm2 = np.arange(cols - shared, cols - shared + cols, dtype=np.int32)
    sch = Schema([Source(S1, idx1, cm1), Source(S2, idx2, cm2)], r_T, c_T, name="config3")
    sch.extras["w_star"] = rng.standard_normal(c_T)
    sch.extras["noise"] = 0.01 * rng.standard_normal(r_T)
    sch.extras["lr"] = np.array([0.1])
    sch.extras["iters"] = np.array([10])
    return sch


def config4(seed: int = 4, r_S: int = 1_000_000, r_R: int = 100_000, c_R: int = 200,
            models: int = 256) -> Schema:
    """Hyper-parameter sweep: ``models`` linear regressions at log-spaced learning rates.

    Draw order: S, R, fk, w_star, noise (sigma 0.01).
    """
    rng = rng_for(seed)
    sch = star_schema(rng, r_S, 20, [(r_R, c_R, "uniform")], name="config4")
    sch.extras["w_star"] = rng.standard_normal(sch.c_T)
    sch.extras["noise"] = 0.01 * rng.standard_normal(r_S)
    sch.extras["lr"] = np.logspace(-3.0, 0.0, models)
    sch.extras["iters"] = np.array([20])
    return sch


def tiny_random_schema(seed: int, r_T: int = 9, c_T: int = 7, n: int = 3,
                       allow_missing: bool = True, integer_values: bool = False) -> Schema:
    """Small random schema exercising fan-out, unmatched rows, dropped and shared columns."""
    rng = rng_for(seed)
    sources = []
    for _ in range(n):
        r_k = int(rng.integers(1, r_T + 1))
        c_k = int(rng.integers(1, c_T + 1))
        if integer_values:
            D = rng.integers(-4, 5, size=(r_k, c_k)).astype(np.float32)
        else:
            D = _normal32(rng, (r_k, c_k))
        idx = rng.integers(0, r_k, size=r_T, dtype=np.int32)
        if allow_missing:
            idx[rng.random(r_T) < 0.25] = -1
        cm = rng.permutation(c_T)[:c_k].astype(np.int32)
        if allow_missing and c_k > 1:
            cm[rng.random(c_k) < 0.2] = -1
        sources.append(Source(D, idx, cm))
    return Schema(sources, r_T, c_T, name=f"tiny{seed}")


def sparsify(schema: Schema, p: float, seed: int) -> Schema:
    """A copy of ``schema`` whose table cells are set to zero independently with probability ``p`` (the sparsity
    parameter of the paper's synthetic data, Tab. 3); index arrays and column maps are shared with the original.
    Draw order: one uniform matrix per source, in source order."""
    rng = rng_for(seed)
    sources = []
    for s in schema.sources:
        D = s.D.copy()
        D[rng.random(D.shape) < p] = 0.0
        sources.append(Source(D, s.row_idx, s.col_map))
    out = Schema(sources, schema.r_T, schema.c_T, name=f"{schema.name}_p{p}")
    out.extras.update(schema.extras)
    return out


@dataclass
class OneHotTable:
    """A dimension table of one-hot encoded attributes in compressed sparse rows, with the rows of the target table
    that join each of its rows (``row_idx``) and its block of target columns (``col_map``)."""
    rowptr: np.ndarray                  # int32 [rows + 1]
    col: np.ndarray                     # int32 [nnz], ascending within a row
    val: np.ndarray                     # float32 [nnz]
    rows: int
    cols: int
    row_idx: np.ndarray                 # int32 [r_T]
    col_map: np.ndarray                 # int32 [cols]

    def dense(self) -> np.ndarray:
        D = np.zeros((self.rows, self.cols), dtype=np.float32)
        r = np.repeat(np.arange(self.rows), np.diff(self.rowptr))
        D[r, self.col] = self.val
        return D


# Shape of the "Movie" row of the paper's table of real data sets (Tab. 4): r_T, then (rows, columns) of the two
# joined tables.  The data themselves are not available here; one_hot_star draws a stand-in of this shape.
MOVIE_SHAPE = (1_000_000, ((6_040, 9_510), (3_710, 3_840)))


def one_hot_star(seed: int, r_T: int, dims, attributes: int = 20):
    """Joined dimension tables of one-hot style: every row of a table has ``attributes`` stored entries, one in each
    of ``attributes`` equal column ranges (a categorical attribute each), all of value 1 except the last, which is
    N(0,1) (a numeric attribute).  Every target row joins one uniformly drawn row of every table.  Target columns are the tables'
    columns side by side; there is no entity table.
    Draw order per table: the column inside each range (rows x attributes integers), the numeric values, the keys."""
    rng = rng_for(seed)
    tables = []
    c0 = 0
    for rows, cols in dims:
        a = min(attributes, cols)
        edges = np.linspace(0, cols, a + 1).astype(np.int64)
        width = np.diff(edges)
        pick = (rng.random((rows, a)) * width[None, :]).astype(np.int64)
        col = (edges[:-1][None, :] + np.minimum(pick, width[None, :] - 1)).astype(np.int32)
        val = np.ones((rows, a), dtype=np.float32)
        val[:, -1] = _normal32(rng, rows)
        rowptr = (np.arange(rows + 1, dtype=np.int64) * a).astype(np.int32)
        fk = rng.integers(0, rows, r_T).astype(np.int32)
        tables.append(OneHotTable(rowptr, col.reshape(-1), val.reshape(-1), rows, cols, fk,
                                  np.arange(c0, c0 + cols, dtype=np.int32)))
        c0 += cols
    return tables, r_T, c0


def finish_labels(kind: str, Tw: np.ndarray, noise: np.ndarray) -> np.ndarray:
    """Labels from a product ``T @ w*`` that the caller computed: ``linear`` adds the noise,
    ``logistic`` thresholds at zero (``sign(0) = +1``) and returns the {0,1} encoding."""
    z = np.asarray(Tw, dtype=np.float64).reshape(-1) + noise
    if kind == "linear":
        return z.astype(np.float32)
    if kind == "logistic":
        return (z >= 0.0).astype(np.float32)
    raise ValueError(kind)
