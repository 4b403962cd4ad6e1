"""CPU oracle for the factorized operators over ``T = sum_k I_k D_k M_k^T``.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the device library is
checked against.  It is imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg, and by nothing on the product path.  It shares no code with the device
library and never calls it.

What it computes (paper, Sec. 2.1 and 2.2):

* the target table by join-gather, i.e. the rewrite rule of Sec. 2.2 with ``X = I``:
  ``T = I_1 D_1 M_1^T + ... + I_n D_n M_n^T`` where ``M_k`` is the mapping matrix of Def. 1 and
  ``I_k`` the indicator matrix of Def. 2;
* on that *materialized* table, in float64: ``T X`` (left multiply, Sec. 2.2), ``T^T Y``
  (the transpose operator Sec. 2.2 names for linear regression), ``T^T T`` and the
  gradient-descent loop of Alg. 1.

Because the rewrite is an identity of linear algebra, the result of every factorized operator
has a plain definition, and the oracle is that definition written out: materialize, then dense
float64 products.  The factorized form appears nowhere in this file.

Readings of the paper taken here (each is also listed in the design document):

* Def. 2 prints the indicator matrix once with the shape of a mapping matrix and once as a "row
  vector of size r_T".  Read: ``I_k`` is logically ``r_T x r_k`` binary with at most one 1 per
  row; the length-``r_T`` vector is its compressed storage (source row, or -1 for none).
* Def. 1: ``M_k`` is ``c_T x c_k`` binary with at most one 1 per row and per column; a source
  column may be unmapped (-1).
* Cells supplied by several sources are summed, literally as the rule of Sec. 2.2 says.
* Alg. 1 prints ``w = w - gamma * X^T((X w) - y)`` with ``X`` the target table.  Read with the
  mean gradient: ``w <- w - gamma * T^T (T w - y) / r_T``; loss ``||T w - y||^2 / (2 r_T)``.
* Logistic regression is only named by the paper (Sec. 3.1, Tab. 7-9).  Read: labels in {0,1},
  ``z = T w``, loss ``mean(softplus(z) - y z)``, gradient ``T^T (sigmoid(z) - y) / r_T``.

* Tab. 2 lists ``T (/) x``, ``f(T)``, ``rowSum(T)`` and ``colSum(T)`` with cost ``m_T`` materialized and
  ``sum_k m_k`` factorized and defines them no further.  Read: ``(/)`` is element-wise arithmetic
  with a scalar ``x`` (times, divide, plus, minus, power), ``f`` an element-wise function (exp, log,
  sqrt, abs, square); both are defined on the cells of the target table, ``rowSum``/``colSum`` are its
  row and column sums.  That the factorized form may apply the operation to every source table
  instead is a property this file does not use; the pins check when it holds (every target cell
  fed by exactly one source cell; for times and divide always).

* KMeans and Gaussian NMF are named among the evaluated models (Sec. 4, Tab. 7-9) and defined nowhere in
  the paper.  Read, for KMeans, one iteration of Lloyd's algorithm on the rows of the target table: every
  row goes to the centroid at the smallest squared Euclidean distance (the first one among equals), every
  centroid becomes the mean of its rows, a centroid without rows stays where it was.  Read, for Gaussian NMF,
  one round of the multiplicative updates of Lee and Seung for ``min ||T - W H||_F^2`` over non-negative
  factors: ``W <- W o (T H^T) / (W H H^T)``, then, with the new ``W``, ``H <- H o (W^T T) / (W^T W H)``
  (``o`` and ``/`` element-wise; a denominator below ``GNMF_TINY`` is raised to it).

Pins (tests/test_oracle_pins.py): brute force from Def. 1 / Def. 2 with dense 0/1 matrices on tiny
schemas; the star-join special case ``T = [S | R[fk]]``; ``T I = T``; ``rowSum``/``colSum`` (Tab. 2);
the adjoint identity; the weighted-Gram closed form of ``T^T T`` for a star join; the closed-form
gradient-descent iterate through an eigendecomposition and its least-squares limit; ``ln 2`` and a
finite-difference gradient for the logistic loss; ``bincount``/stable ``argsort`` for the inverse
index; for KMeans the nearest-centroid and one-iteration routines of ``scipy.cluster.vq``, a loop over
points and centroids on tiny inputs, the group means of well separated blobs and the monotone objective;
for Gaussian NMF one iteration of scikit-learn's multiplicative-update solver, the fixed point at an
exact factorization, an element-by-element loop on tiny inputs and the monotone objective; for the rounding to
bfloat16 torch's conversion and hand-worked ties, for Alg. 1 with rounded product inputs (``gd_bf16_inputs``, the
arithmetic of the reduced-precision variant with exact accumulation) the first iteration on representable inputs,
which must equal Alg. 1's, and the error bound derived for it in tests/tolerances.py.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

ROW_CHUNK = 262_144   # rows converted to float64 at a time; memory bound only, no effect on values


# ----------------------------------------------------------------------------- definitions
def dense_mapping(col_map: np.ndarray, c_T: int) -> np.ndarray:
    """Def. 1: ``M_k[i, j] = 1`` iff source column ``j`` is mapped to target column ``i``."""
    c_k = len(col_map)
    M = np.zeros((c_T, c_k), dtype=np.float64)
    for j in range(c_k):
        i = int(col_map[j])
        if i >= 0:
            M[i, j] = 1.0
    return M


def dense_indicator(row_idx: Optional[np.ndarray], r_T: int, r_k: int) -> np.ndarray:
    """Def. 2: ``I_k[i, j] = 1`` iff source row ``j`` is mapped to target row ``i``."""
    I = np.zeros((r_T, r_k), dtype=np.float64)
    for i in range(r_T):
        j = i if row_idx is None else int(row_idx[i])
        if j >= 0:
            I[i, j] = 1.0
    return I


def brute_force_target(schema) -> np.ndarray:
    """Sec. 2.2 rewrite with ``X = I``, evaluated with dense 0/1 matrices (tiny inputs only)."""
    T = np.zeros((schema.r_T, schema.c_T), dtype=np.float64)
    for s in schema.sources:
        I = dense_indicator(s.row_idx, schema.r_T, s.rows)
        M = dense_mapping(s.col_map, schema.c_T)
        T += I @ s.D.astype(np.float64) @ M.T
    return T


# ----------------------------------------------------------------------------- materialize
def materialize(schema, row_lo: int = 0, row_hi: Optional[int] = None) -> np.ndarray:
    """Join-gather of target rows ``[row_lo, row_hi)`` in float32.

    For every source in order, every target row ``i`` with a source row and every mapped source
    column ``j``: ``T[i, col_map[j]] += D_k[row_idx[i], j]`` starting from ``+0.0``.  This float32
    table is the bit-exact expectation for the device join-gather.
    """
    row_hi = schema.r_T if row_hi is None else row_hi
    n = row_hi - row_lo
    T = np.zeros((n, schema.c_T), dtype=np.float32)
    for s in schema.sources:
        if s.row_idx is None:
            src_rows = np.arange(row_lo, row_hi, dtype=np.int64)
        else:
            src_rows = s.row_idx[row_lo:row_hi].astype(np.int64)
        present = np.flatnonzero(src_rows >= 0)
        if present.size == 0:
            continue
        picked = src_rows[present]
        for j in range(s.cols):
            t = int(s.col_map[j])
            if t < 0:
                continue
            T[present, t] += s.D[picked, j]
    return T


def _chunks(r_T: int):
    for lo in range(0, r_T, ROW_CHUNK):
        yield lo, min(r_T, lo + ROW_CHUNK)


class Target:
    """The materialized float32 target table, held once, widened to float64 chunk by chunk."""

    def __init__(self, schema=None, table: Optional[np.ndarray] = None):
        if table is None:
            table = np.empty((schema.r_T, schema.c_T), dtype=np.float32)
            for lo, hi in _chunks(schema.r_T):
                table[lo:hi] = materialize(schema, lo, hi)
        self.T32 = table
        self.r_T, self.c_T = table.shape

    def rows64(self, lo: int, hi: int) -> np.ndarray:
        return self.T32[lo:hi].astype(np.float64)


def _as_target(obj) -> Target:
    return obj if isinstance(obj, Target) else Target(obj)


# ----------------------------------------------------------------------------- operators
def lmm(target, X: np.ndarray) -> np.ndarray:
    """Left multiply ``T X`` (Sec. 2.2), float64, ``X`` is ``c_T x c_X``."""
    tg = _as_target(target)
    X64 = np.asarray(X, dtype=np.float64).reshape(tg.c_T, -1)
    out = np.empty((tg.r_T, X64.shape[1]), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out[lo:hi] = tg.rows64(lo, hi) @ X64
    return out


def tmm(target, Y: np.ndarray) -> np.ndarray:
    """Transposed multiply ``T^T Y``, float64, ``Y`` is ``r_T x c_X``."""
    tg = _as_target(target)
    Y64 = np.asarray(Y, dtype=np.float64).reshape(tg.r_T, -1)
    out = np.zeros((tg.c_T, Y64.shape[1]), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out += tg.rows64(lo, hi).T @ Y64[lo:hi]
    return out


def rmm(target, X: np.ndarray) -> np.ndarray:
    """Right multiply ``X T`` (Tab. 2, row ``XT``), float64, ``X`` is ``r_X x r_T``."""
    tg = _as_target(target)
    X64 = np.asarray(X, dtype=np.float64).reshape(-1, tg.r_T)
    out = np.zeros((X64.shape[0], tg.c_T), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out += X64[:, lo:hi] @ tg.rows64(lo, hi)
    return out


def crossprod(target) -> np.ndarray:
    """Gram matrix ``T^T T``, float64, full symmetric ``c_T x c_T``."""
    tg = _as_target(target)
    out = np.zeros((tg.c_T, tg.c_T), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        blk = tg.rows64(lo, hi)
        out += blk.T @ blk
    return out


# ----------------------------------------------------------------------------- inverse index
def inverse_index(row_idx: np.ndarray, r_k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Compressed-row form of ``I_k^T``: for each source row the target rows it feeds, ascending.

    Returns ``(rowptr int32[r_k+1], perm int32[nnz], cnt int32[r_k])``.  Written as the definition:
    walk the target rows in order and append each to the list of its source row.
    """
    lists: List[List[int]] = [[] for _ in range(r_k)]
    for i, j in enumerate(np.asarray(row_idx).tolist()):
        if j >= 0:
            lists[j].append(i)
    cnt = np.array([len(l) for l in lists], dtype=np.int32)
    rowptr = np.zeros(r_k + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(cnt)
    perm = np.array([i for l in lists for i in l], dtype=np.int32)
    return rowptr, perm, cnt


def segment_sum(row_idx: np.ndarray, r_k: int, Y: np.ndarray) -> np.ndarray:
    """``I_k^T Y`` from the dense definition of ``I_k`` chunked over target rows, float64."""
    Y64 = np.asarray(Y, dtype=np.float64).reshape(len(row_idx), -1)
    Z = np.zeros((r_k, Y64.shape[1]), dtype=np.float64)
    for i, j in enumerate(np.asarray(row_idx).tolist()):
        if j >= 0:
            Z[j] += Y64[i]
    return Z


# ----------------------------------------------------------------------------- gradient descent
def linear_loss_grad(target, y: np.ndarray, W: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Loss ``||T w - y||^2 / (2 r_T)`` and gradient ``T^T (T w - y) / r_T`` per column of ``W``."""
    tg = _as_target(target)
    W = np.asarray(W, dtype=np.float64).reshape(tg.c_T, -1)
    y64 = np.asarray(y, dtype=np.float64).reshape(-1, 1)
    loss = np.zeros(W.shape[1])
    grad = np.zeros_like(W)
    for lo, hi in _chunks(tg.r_T):
        blk = tg.rows64(lo, hi)
        e = blk @ W - y64[lo:hi]
        loss += 0.5 * np.sum(e * e, axis=0)
        grad += blk.T @ e
    return loss / tg.r_T, grad / tg.r_T


def _softplus(z: np.ndarray) -> np.ndarray:
    return np.maximum(z, 0.0) + np.log1p(np.exp(-np.abs(z)))


def _sigmoid(z: np.ndarray) -> np.ndarray:
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def logistic_loss_grad(target, y01: np.ndarray, W: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Mean cross-entropy ``mean(softplus(z) - y z)`` with ``z = T w`` and its gradient
    ``T^T (sigmoid(z) - y) / r_T``; labels in {0, 1}."""
    tg = _as_target(target)
    W = np.asarray(W, dtype=np.float64).reshape(tg.c_T, -1)
    y64 = np.asarray(y01, dtype=np.float64).reshape(-1, 1)
    loss = np.zeros(W.shape[1])
    grad = np.zeros_like(W)
    for lo, hi in _chunks(tg.r_T):
        blk = tg.rows64(lo, hi)
        z = blk @ W
        loss += np.sum(_softplus(z) - y64[lo:hi] * z, axis=0)
        grad += blk.T @ (_sigmoid(z) - y64[lo:hi])
    return loss / tg.r_T, grad / tg.r_T


def gd(target, model: str, y: np.ndarray, W0: np.ndarray, lr: Sequence[float], iters: int):
    """Alg. 1 for ``iters`` iterations: ``W <- W - grad * diag(lr)``, one learning rate per column.

    Returns the final weights and the per-iteration loss measured *before* each update.
    """
    tg = _as_target(target)
    W = np.array(W0, dtype=np.float64).reshape(tg.c_T, -1).copy()
    lr64 = np.asarray(lr, dtype=np.float64).reshape(1, -1)
    fn = {"linear": linear_loss_grad, "logistic": logistic_loss_grad}[model]
    losses = []
    for _ in range(iters):
        loss, grad = fn(tg, y, W)
        losses.append(loss)
        W -= grad * lr64
    return W, np.array(losses)


# ----------------------------------------------------------------------------- bfloat16-input variant of Alg. 1
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Values rounded to the nearest number with 8 significant bits (bfloat16: sign, 8 exponent bits,
    7 stored mantissa bits), ties to the even neighbour, returned as float64.  Works on the float32 bit
    pattern: the input is first rounded to float32, as the device holds it."""
    f32 = np.ascontiguousarray(a, dtype=np.float32)
    bits = f32.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(f32.shape).astype(np.float64)


def gd_bf16_inputs(target, model: str, y: np.ndarray, W0: np.ndarray, lr: Sequence[float], iters: int):
    """Alg. 1 with both factors of every product rounded to bfloat16 as they enter it and everything else
    exact: ``z = rd(T) rd(W)``, residual ``e`` (``z - y`` or ``sigmoid(z) - y``) and loss from the unrounded
    ``z``, gradient ``rd(T)^T rd(e) / r_T``, weights kept unrounded between iterations.  This is the arithmetic
    of the reduced-precision variant with exact accumulation; it exists to check the tolerance that the tests
    of that variant use against Alg. 1 in full precision (``gd``).  Returns weights and per-iteration losses."""
    tg = _as_target(target)
    W = np.array(W0, dtype=np.float64).reshape(tg.c_T, -1).copy()
    lr64 = np.asarray(lr, dtype=np.float64).reshape(1, -1)
    y64 = np.asarray(y, dtype=np.float64).reshape(-1, 1)
    losses = []
    for _ in range(iters):
        Wr = round_to_bf16(W)
        loss = np.zeros(W.shape[1])
        grad = np.zeros_like(W)
        for lo, hi in _chunks(tg.r_T):
            blk = round_to_bf16(tg.T32[lo:hi])
            z = blk @ Wr
            if model == "linear":
                e = z - y64[lo:hi]
                loss += 0.5 * np.sum(e * e, axis=0)
            else:
                e = _sigmoid(z) - y64[lo:hi]
                loss += np.sum(_softplus(z) - y64[lo:hi] * z, axis=0)
            grad += blk.T @ round_to_bf16(e)
        losses.append(loss / tg.r_T)
        W -= (grad / tg.r_T) * lr64
    return W, np.array(losses)


# ----------------------------------------------------------------------------- complexity (Tab. 2)
def complexity_lmm(schema, c_X: int) -> Tuple[int, int]:
    """Tab. 2 row ``T X``: (materialized, factorized) operation counts for dense operands."""
    m_T = schema.r_T * schema.c_T
    m_X = schema.c_T * c_X
    mat = c_X * m_T + schema.r_T * m_X
    fact = sum(c_X * s.rows * s.cols + s.rows * m_X for s in schema.sources)
    return mat, fact


# ----------------------------------------------------------------------------- scalar operators (Tab. 2)
ELEMENTWISE_OPS = ("mul", "div", "add", "sub", "pow", "exp", "log", "sqrt", "abs", "square")


def apply_elementwise(A: np.ndarray, op: str, x: float = 0.0) -> np.ndarray:
    """``A (/) x`` or ``f(A)`` cell by cell in float64 (Tab. 2, first two rows)."""
    A = np.asarray(A, dtype=np.float64)
    if op == "mul":
        return A * x
    if op == "div":
        return A / x
    if op == "add":
        return A + x
    if op == "sub":
        return A - x
    if op == "pow":
        return np.power(A, x)
    if op == "exp":
        return np.exp(A)
    if op == "log":
        return np.log(A)
    if op == "sqrt":
        return np.sqrt(A)
    if op == "abs":
        return np.abs(A)
    if op == "square":
        return A * A
    raise ValueError(op)


def elementwise(target, op: str, x: float = 0.0) -> np.ndarray:
    """The element-wise operators of Tab. 2 on the materialized table, float64, ``r_T x c_T``."""
    tg = _as_target(target)
    out = np.empty((tg.r_T, tg.c_T), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out[lo:hi] = apply_elementwise(tg.rows64(lo, hi), op, x)
    return out


def row_sum(target) -> np.ndarray:
    """``rowSum(T)`` (Tab. 2): float64 vector of length ``r_T``."""
    tg = _as_target(target)
    out = np.empty(tg.r_T, dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out[lo:hi] = tg.rows64(lo, hi).sum(axis=1)
    return out


def col_sum(target) -> np.ndarray:
    """``colSum(T)`` (Tab. 2): float64 vector of length ``c_T``."""
    tg = _as_target(target)
    out = np.zeros(tg.c_T, dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        out += tg.rows64(lo, hi).sum(axis=0)
    return out


def cover_counts(schema) -> np.ndarray:
    """How many source cells feed each target cell: ``sum_k I_k 1 1^T M_k^T`` (Def. 1, Def. 2), int64
    ``r_T x c_T``.  The factorized element-wise operators need every count to be exactly one."""
    C = np.zeros((schema.r_T, schema.c_T), dtype=np.int64)
    for s in schema.sources:
        if s.D.shape[0] == 0 or s.D.shape[1] == 0:
            continue
        rows = np.arange(schema.r_T) if s.row_idx is None else np.flatnonzero(np.asarray(s.row_idx) >= 0)
        cols = np.asarray(s.col_map)[np.asarray(s.col_map) >= 0]
        C[np.ix_(rows, cols)] += 1
    return C


# ----------------------------------------------------------------------------- cost analysis (Sec. 3)
def complexity_rmm(schema, r_X: int) -> Tuple[int, int]:
    """Tab. 2 row ``X T``: (materialized, factorized) operation counts for a dense ``r_X x r_T`` operand:
    ``r_X m_T + c_T m_X`` against ``sum_k (r_X m_k + c_k m_X)``."""
    m_T = schema.r_T * schema.c_T
    m_X = r_X * schema.r_T
    mat = r_X * m_T + schema.c_T * m_X
    fact = sum(r_X * s.D.shape[0] * s.D.shape[1] + s.D.shape[1] * m_X for s in schema.sources)
    return mat, fact


def complexity_lr(schema) -> Tuple[int, int]:
    """Sec. 3.1, linear regression with dense operands: ``(O_materialized, O_factorized)``.
    ``w`` is ``c_T x 1`` (``c_w = 1``, ``m_w = c_T``) and ``X = T w`` is ``r_T x 1`` (``m_X = r_T``):
    ``O_mat = (c_w m_T + r_T m_w) + (m_T + c_T m_X)`` and
    ``O_fact = sum_k (c_w m_k + r_k m_w) + sum_k (m_k + c_k m_X)``."""
    r_T, c_T = schema.r_T, schema.c_T
    m_T, m_w, m_X, c_w = r_T * c_T, c_T, r_T, 1
    o_mat = (c_w * m_T + r_T * m_w) + (m_T + c_T * m_X)
    o_fact = 0
    for s in schema.sources:
        r_k, c_k = s.D.shape
        m_k = r_k * c_k
        o_fact += (c_w * m_k + r_k * m_w) + (m_k + c_k * m_X)
    return o_mat, o_fact


def tuple_and_feature_ratio(schema) -> Tuple[float, float]:
    """The redundancy measures Sec. 4.3 compares with (thresholds 5 and 1): target rows per row of the joined
    tables and joined columns per column of the base table.  Read for several tables: sums over the sources
    that are joined through a row index, against the sources that are not."""
    joined = [s for s in schema.sources if s.row_idx is not None]
    base = [s for s in schema.sources if s.row_idx is None]
    rows = sum(s.D.shape[0] for s in joined)
    tr = schema.r_T / rows if rows else 0.0
    bc = sum(s.D.shape[1] for s in base)
    fr = sum(s.D.shape[1] for s in joined) / bc if bc else 0.0
    return tr, fr


# ----------------------------------------------------------------------------- KMeans, Gaussian NMF (named in Sec. 4; see the readings above)
GNMF_TINY = 1e-30


def kmeans_distances(target, C: np.ndarray) -> np.ndarray:
    """Squared Euclidean distance of every target row to every centroid; ``C`` is ``c_T x k``, column j = centroid j."""
    tg = _as_target(target)
    C64 = np.asarray(C, dtype=np.float64).reshape(tg.c_T, -1)
    d2 = np.empty((tg.r_T, C64.shape[1]), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        blk = tg.rows64(lo, hi)
        for j in range(C64.shape[1]):
            diff = blk - C64[:, j][None, :]
            d2[lo:hi, j] = np.sum(diff * diff, axis=1)
    return d2


def kmeans_step(target, C: np.ndarray):
    """One Lloyd iteration.  Returns the new centroids (``c_T x k``), the assignment of every row (to the old
    centroids), the cluster sizes and the sum of squared distances to the assigned old centroids."""
    tg = _as_target(target)
    C64 = np.asarray(C, dtype=np.float64).reshape(tg.c_T, -1)
    k = C64.shape[1]
    d2 = kmeans_distances(tg, C64)
    assign = np.argmin(d2, axis=1).astype(np.int32)          # argmin returns the first of equal minima
    counts = np.bincount(assign, minlength=k).astype(np.int64)
    sums = np.zeros((tg.c_T, k), dtype=np.float64)
    for lo, hi in _chunks(tg.r_T):
        blk = tg.rows64(lo, hi)
        for j in range(k):
            sums[:, j] += blk[assign[lo:hi] == j].sum(axis=0)
    C_new = C64.copy()
    for j in range(k):
        if counts[j] > 0:
            C_new[:, j] = sums[:, j] / counts[j]
    inertia = float(np.sum(d2[np.arange(tg.r_T), assign]))
    return C_new, assign, counts, inertia


def gnmf_objective(target, W: np.ndarray, H: np.ndarray) -> float:
    """``||T - W H||_F^2 / 2`` for ``W`` (``r_T x r``) and ``H`` (``r x c_T``)."""
    tg = _as_target(target)
    W64 = np.asarray(W, dtype=np.float64)
    H64 = np.asarray(H, dtype=np.float64)
    total = 0.0
    for lo, hi in _chunks(tg.r_T):
        res = tg.rows64(lo, hi) - W64[lo:hi] @ H64
        total += float(np.sum(res * res))
    return 0.5 * total


def gnmf_step(target, W: np.ndarray, H: np.ndarray):
    """One round of multiplicative updates: first ``W`` (with the old ``H``), then ``H`` (with the new ``W``)."""
    tg = _as_target(target)
    W64 = np.asarray(W, dtype=np.float64).reshape(tg.r_T, -1)
    H64 = np.asarray(H, dtype=np.float64).reshape(-1, tg.c_T)
    TH = lmm(tg, H64.T)                                       # T H^T, r_T x r
    W1 = W64 * TH / np.maximum(W64 @ (H64 @ H64.T), GNMF_TINY)
    WtT = tmm(tg, W1).T                                       # W^T T, r x c_T
    H1 = H64 * WtT / np.maximum((W1.T @ W1) @ H64, GNMF_TINY)
    return W1, H1
