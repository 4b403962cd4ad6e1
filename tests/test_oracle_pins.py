"""Pins for the CPU oracle: every check compares it with something other than itself.

Sources of truth used here: the dense 0/1 matrices of Def. 1 and Def. 2 multiplied out as the
rewrite rule of Sec. 2.2 says (brute force on tiny schemas), numpy library routines on special
cases (fancy indexing for a star join, bincount, stable argsort, lstsq, eigh), algebraic
identities (adjoint, trace, x^T G x = |T x|^2) and closed forms for gradient descent.
"""
import numpy as np
import pytest

import datagen
import oracle

TINY_SEEDS = list(range(12))


def _factorized_lmm_fp64(schema, X):
    """The rewritten form  sum_k I_k (D_k (M_k^T X))  spelled out with index arrays, for the identity test."""
    X = np.asarray(X, dtype=np.float64)
    out = np.zeros((schema.r_T, X.shape[1]))
    for s in schema.sources:
        keep = np.flatnonzero(s.col_map >= 0)
        P = s.D[:, keep].astype(np.float64) @ X[s.col_map[keep]]
        if s.row_idx is None:
            out += P
        else:
            ok = np.flatnonzero(s.row_idx >= 0)
            out[ok] += P[s.row_idx[ok]]
    return out


# ------------------------------------------------------------------ materialize
@pytest.mark.parametrize("seed", TINY_SEEDS)
def test_materialize_equals_dense_definition_bit_exact(seed):
    # integer-valued tables: every partial sum is exact, so float32 join-gather must equal the
    # float64 triple products of the 0/1 matrices bit for bit, shared columns included
    sch = datagen.tiny_random_schema(seed, r_T=11, c_T=8, n=3, integer_values=True)
    want = oracle.brute_force_target(sch)
    got = oracle.materialize(sch)
    assert got.dtype == np.float32
    assert np.array_equal(got.astype(np.float64), want)


@pytest.mark.parametrize("seed", TINY_SEEDS)
def test_materialize_equals_dense_definition_real_values(seed):
    sch = datagen.tiny_random_schema(100 + seed, r_T=12, c_T=6, n=3)
    want = oracle.brute_force_target(sch)
    got = oracle.materialize(sch).astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=0, atol=4e-7 * max(1.0, np.abs(want).max()))
    # cells fed by at most one source are copies: exact
    feeders = np.zeros((sch.r_T, sch.c_T), dtype=int)
    for s in sch.sources:
        rows = np.flatnonzero(s.row_idx >= 0)
        cols = s.col_map[s.col_map >= 0]
        feeders[np.ix_(rows, cols)] += 1
    single = feeders <= 1
    assert np.array_equal(got[single], want[single])
    assert np.all(got[feeders == 0] == 0.0)


def test_materialize_star_join_is_hstack():
    sch = datagen.config0()
    S, R = sch.sources[0].D, sch.sources[1].D
    fk = sch.sources[1].row_idx
    want = np.hstack([S, R[fk]])
    got = oracle.materialize(sch)
    assert got.shape == (10_000, 12)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_materialize_row_ranges_tile_the_table():
    sch = datagen.config3(rows=500, cols=8, shared=4)
    full = oracle.materialize(sch)
    parts = [oracle.materialize(sch, lo, min(lo + 137, sch.r_T)) for lo in range(0, sch.r_T, 137)]
    assert np.array_equal(np.vstack(parts), full)


def test_union_config_structure():
    sch = datagen.config3(rows=1000, cols=8, shared=4)
    assert sch.r_T == 1700 and sch.c_T == 12
    T = oracle.materialize(sch)
    S1, S2 = sch.sources[0].D, sch.sources[1].D
    idx2 = sch.sources[1].row_idx
    # S1 rows occupy the first block, their shared cells come from S1 alone
    assert np.array_equal(T[:1000, :8], S1)
    matched = np.flatnonzero(idx2[:1000] >= 0)
    assert matched.size == 300
    assert np.array_equal(T[matched, 8:], S2[idx2[matched], 4:])
    # the new S2 rows carry zeros in the S1-only block
    assert np.all(T[1000:, :4] == 0)
    assert np.array_equal(T[1000:, 4:], S2[idx2[1000:]])


# ------------------------------------------------------------------ LMM
@pytest.mark.parametrize("seed", TINY_SEEDS[:6])
def test_lmm_tiny_equals_dense_definition(seed):
    sch = datagen.tiny_random_schema(200 + seed, n=3)
    X = datagen.rng_for(seed).standard_normal((sch.c_T, 3))
    # the brute-force target shares columns between sources in float64; the oracle adds them in
    # float32 first, hence the tolerance
    np.testing.assert_allclose(oracle.lmm(sch, X), oracle.brute_force_target(sch) @ X, rtol=0, atol=1e-5)


def test_lmm_identity_and_rowsum():
    sch = datagen.config0(r_S=777, r_R=50)
    T = oracle.materialize(sch).astype(np.float64)
    assert np.array_equal(oracle.lmm(sch, np.eye(sch.c_T)), T)
    np.testing.assert_allclose(oracle.lmm(sch, np.ones((sch.c_T, 1)))[:, 0], T.sum(axis=1), rtol=1e-13)


@pytest.mark.parametrize("maker", [
    lambda: datagen.config0(),
    lambda: datagen.config2(r_S=4000, dim_rows=(100, 50, 10)),
    lambda: datagen.config3(rows=900, cols=16, shared=8),
    lambda: datagen.tiny_random_schema(5, r_T=40, c_T=9, n=4),
])
def test_factorized_form_equals_materialized_form(maker):
    sch = maker()
    X = datagen.rng_for(9).standard_normal((sch.c_T, 5))
    want = _factorized_lmm_fp64(sch, X)
    got = oracle.lmm(sch, X)
    # shared target cells are added in float32 by the join-gather, in float64 by the rewritten form
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-6 * np.abs(want).max())


# ------------------------------------------------------------------ TMM
def test_tmm_adjoint_identity():
    sch = datagen.config2(r_S=3000, dim_rows=(120, 60, 10))
    rng = datagen.rng_for(3)
    X = rng.standard_normal((sch.c_T, 4))
    Y = rng.standard_normal((sch.r_T, 4))
    lhs = np.sum(oracle.lmm(sch, X) * Y)
    rhs = np.sum(X * oracle.tmm(sch, Y))
    assert abs(lhs - rhs) <= 1e-10 * max(abs(lhs), 1.0)


def test_tmm_colsum_and_unit_vectors():
    sch = datagen.config3(rows=300, cols=8, shared=4)
    T = oracle.materialize(sch).astype(np.float64)
    np.testing.assert_allclose(oracle.tmm(sch, np.ones((sch.r_T, 1)))[:, 0], T.sum(axis=0), rtol=1e-12, atol=1e-12)
    for i in (0, 299, 300, sch.r_T - 1):
        e = np.zeros((sch.r_T, 1)); e[i] = 1.0
        assert np.array_equal(oracle.tmm(sch, e)[:, 0], T[i])


def test_tmm_not_transposed_operand():
    # a non-square case where T X and T^T Y cannot be confused
    sch = datagen.tiny_random_schema(7, r_T=13, c_T=5, n=2)
    T = oracle.brute_force_target(sch)
    Y = datagen.rng_for(1).standard_normal((13, 2))
    np.testing.assert_allclose(oracle.tmm(sch, Y), T.T @ Y, atol=1e-5)


# ------------------------------------------------------------------ segment sum / inverse index
def test_segment_sum_equals_bincount():
    rng = datagen.rng_for(11)
    r_k, r_T = 37, 1000
    idx = rng.integers(-1, r_k, size=r_T).astype(np.int32)
    Y = rng.standard_normal((r_T, 3))
    got = oracle.segment_sum(idx, r_k, Y)
    ok = idx >= 0
    for c in range(3):
        want = np.bincount(idx[ok], weights=Y[ok, c], minlength=r_k)
        np.testing.assert_allclose(got[:, c], want, rtol=1e-12, atol=1e-12)
    cnt = oracle.segment_sum(idx, r_k, np.ones((r_T, 1)))[:, 0]
    assert np.array_equal(cnt, np.bincount(idx[ok], minlength=r_k))


def test_inverse_index_is_stable_grouping():
    rng = datagen.rng_for(12)
    r_k, r_T = 23, 500
    idx = rng.integers(-1, r_k + 0, size=r_T).astype(np.int32)
    idx[idx == 5] = 6            # an empty segment
    rowptr, perm, cnt = oracle.inverse_index(idx, r_k)
    valid = np.flatnonzero(idx >= 0)
    order = valid[np.argsort(idx[valid], kind="stable")]
    assert np.array_equal(perm, order.astype(np.int32))
    assert np.array_equal(cnt, np.bincount(idx[valid], minlength=r_k))
    assert rowptr[0] == 0 and rowptr[-1] == valid.size and np.all(np.diff(rowptr) == cnt)
    assert cnt[5] == 0
    for j in range(r_k):
        seg = perm[rowptr[j]:rowptr[j + 1]]
        assert np.all(idx[seg] == j) and np.all(np.diff(seg) > 0)


# ------------------------------------------------------------------ crossprod
def test_crossprod_identities():
    sch = datagen.config3(rows=400, cols=8, shared=4)
    G = oracle.crossprod(sch)
    T = oracle.materialize(sch)
    np.testing.assert_allclose(G, oracle.tmm(sch, T), rtol=1e-12, atol=1e-10)
    assert np.array_equal(G, G.T)
    assert abs(np.trace(G) - np.sum(T.astype(np.float64) ** 2)) < 1e-9 * np.trace(G)
    assert np.linalg.eigvalsh(G).min() >= -1e-9 * np.trace(G)
    x = datagen.rng_for(2).standard_normal((sch.c_T, 1))
    q = (x.T @ G @ x).item()
    assert abs(q - float(np.sum(oracle.lmm(sch, x) ** 2))) < 1e-9 * q


def test_crossprod_star_closed_form():
    sch = datagen.config0(r_S=2000, r_R=64)
    S = sch.sources[0].D.astype(np.float64)
    R = sch.sources[1].D.astype(np.float64)
    fk = sch.sources[1].row_idx
    cnt = np.bincount(fk, minlength=64).astype(np.float64)
    seg = np.zeros((64, 4))
    np.add.at(seg, fk, S)
    want = np.block([[S.T @ S, seg.T @ R], [R.T @ seg, R.T @ (cnt[:, None] * R)]])
    np.testing.assert_allclose(oracle.crossprod(sch), want, rtol=1e-11, atol=1e-9)


# ------------------------------------------------------------------ linear regression (Alg. 1)
def _config0_problem():
    sch = datagen.config0()
    tg = oracle.Target(sch)
    y = datagen.finish_labels("linear", oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])
    return sch, tg, y


def test_linear_gd_matches_closed_form_iterate():
    sch, tg, y = _config0_problem()
    T = tg.T32.astype(np.float64)
    y64 = y.astype(np.float64)
    gamma, iters = 0.1, 20
    W, losses = oracle.gd(tg, "linear", y, np.zeros((12, 1)), [gamma], iters)
    w_ls = np.linalg.lstsq(T, y64, rcond=None)[0]
    H = T.T @ T / sch.r_T
    lam, Q = np.linalg.eigh(H)
    assert gamma * lam.max() < 2.0
    # w_t - w_ls = (I - gamma H)^t (w_0 - w_ls)
    w_t = w_ls + Q @ (((1.0 - gamma * lam) ** iters) * (Q.T @ (0.0 - w_ls)))
    np.testing.assert_allclose(W[:, 0], w_t, rtol=0, atol=1e-11)
    assert np.all(np.diff(losses[:, 0]) < 0)
    # loss before the first update is |y|^2 / (2 r_T)
    assert abs(losses[0, 0] - 0.5 * np.mean(y64 ** 2)) < 1e-12 * losses[0, 0]
    # after 20 iterations the iterate is still visibly away from the optimum: trajectory, not limit
    assert 0.02 < np.linalg.norm(W[:, 0] - w_ls) / np.linalg.norm(w_ls) < 0.3


def test_linear_gd_converges_to_least_squares():
    sch, tg, y = _config0_problem()
    T = tg.T32.astype(np.float64)
    w_ls = np.linalg.lstsq(T, y.astype(np.float64), rcond=None)[0]
    W, _ = oracle.gd(tg, "linear", y, np.zeros((12, 1)), [1.0], 400)
    assert np.linalg.norm(W[:, 0] - w_ls) / np.linalg.norm(w_ls) < 1e-10
    # the optimum sits within the noise floor of the generating weights
    assert np.linalg.norm(w_ls - sch.extras["w_star"]) < 10 * 0.01 * np.sqrt(12 / 10_000)


def test_linear_gd_one_learning_rate_per_column():
    sch = datagen.config0(r_S=500, r_R=20)
    tg = oracle.Target(sch)
    y = datagen.finish_labels("linear", oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])
    lrs = [0.05, 0.3, 1.0]
    W, L = oracle.gd(tg, "linear", y, np.zeros((12, 3)), lrs, 7)
    for c, g in enumerate(lrs):
        Wc, Lc = oracle.gd(tg, "linear", y, np.zeros((12, 1)), [g], 7)
        np.testing.assert_allclose(W[:, c], Wc[:, 0], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(L[:, c], Lc[:, 0], rtol=1e-13)


# ------------------------------------------------------------------ logistic regression
def _small_logistic():
    sch = datagen.config2(r_S=3000, dim_rows=(100, 50, 10))
    tg = oracle.Target(sch)
    y01 = datagen.finish_labels("logistic", oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])
    return sch, tg, y01


def test_logistic_at_zero_weights():
    sch, tg, y01 = _small_logistic()
    loss, grad = oracle.logistic_loss_grad(tg, y01, np.zeros((sch.c_T, 1)))
    assert abs(loss[0] - np.log(2.0)) < 1e-15
    T = tg.T32.astype(np.float64)
    np.testing.assert_allclose(grad[:, 0], T.T @ (0.5 - y01.astype(np.float64)) / sch.r_T, rtol=1e-12, atol=1e-15)
    assert set(np.unique(y01)) == {0.0, 1.0}


def test_logistic_gradient_finite_difference():
    sch, tg, y01 = _small_logistic()
    rng = datagen.rng_for(5)
    w = 0.3 * rng.standard_normal((sch.c_T, 1))
    _, grad = oracle.logistic_loss_grad(tg, y01, w)
    h = 1e-6
    for j in rng.choice(sch.c_T, size=12, replace=False):
        d = np.zeros_like(w); d[j] = h
        lp, _ = oracle.logistic_loss_grad(tg, y01, w + d)
        lm, _ = oracle.logistic_loss_grad(tg, y01, w - d)
        assert abs((lp[0] - lm[0]) / (2 * h) - grad[j, 0]) < 1e-8


def test_logistic_loss_matches_plus_minus_one_form_and_decreases():
    sch, tg, y01 = _small_logistic()
    rng = datagen.rng_for(6)
    w = 0.2 * rng.standard_normal((sch.c_T, 1))
    loss, _ = oracle.logistic_loss_grad(tg, y01, w)
    z = (tg.T32.astype(np.float64) @ w)[:, 0]
    ypm = 2.0 * y01.astype(np.float64) - 1.0
    assert abs(loss[0] - np.mean(np.log1p(np.exp(-ypm * z)))) < 1e-12
    # 50 Zipf keys put a quarter of the rows on one key: the curvature bound needs a small step here
    _, losses = oracle.gd(tg, "logistic", y01, np.zeros((sch.c_T, 1)), [0.05], 15)
    assert np.all(np.diff(losses[:, 0]) < 0)


def test_logistic_stable_for_large_logits():
    T = np.array([[800.0], [-800.0]], dtype=np.float32)
    tg = oracle.Target(table=T)
    loss, grad = oracle.logistic_loss_grad(tg, np.array([1.0, 0.0]), np.ones((1, 1)))
    assert np.isfinite(loss[0]) and loss[0] < 1e-300 + 1e-12
    assert np.all(np.isfinite(grad))


# ------------------------------------------------------------------ generators
def test_zipf_keys_head_mass():
    rng = datagen.rng_for(2)
    keys = datagen.bounded_zipf_keys(rng, 400_000, 50_000, 1.1)
    cnt = np.sort(np.bincount(keys, minlength=50_000))[::-1]
    H = np.sum(np.arange(1, 50_001, dtype=np.float64) ** -1.1)
    assert abs(cnt[0] / 400_000 - 1.0 / H) < 0.01
    assert abs(cnt[1] / cnt[0] - 2 ** -1.1) < 0.03


def test_generators_are_seeded():
    a, b = datagen.config0(), datagen.config0()
    assert all(np.array_equal(x.D, y.D) for x, y in zip(a.sources, b.sources))
    assert np.array_equal(a.sources[1].row_idx, b.sources[1].row_idx)
    c = datagen.config0(seed=5)
    assert not np.array_equal(a.sources[0].D, c.sources[0].D)


def test_complexity_formula_tab2():
    sch = datagen.config1(r_S=1000, r_R=100, c_R=200)
    mat, fact = oracle.complexity_lmm(sch, 1)
    assert mat == 1 * 1000 * 220 + 1000 * 220
    assert fact == (1000 * 20 + 1000 * 220) + (100 * 200 + 100 * 220)


# ----------------------------------------------------------------------------- scalar operators (Tab. 2)
def _assemble_dense(schema, tables):
    """sum_k I_k A_k M_k^T with the dense 0/1 matrices of Def. 1 / Def. 2 and the given per-source tables."""
    out = np.zeros((schema.r_T, schema.c_T))
    for s, A in zip(schema.sources, tables):
        I = oracle.dense_indicator(s.row_idx, schema.r_T, s.D.shape[0])
        M = oracle.dense_mapping(s.col_map, schema.c_T)
        out += I @ np.asarray(A, dtype=np.float64) @ M.T
    return out


def _star(seed, r_T=23, positive=False):
    rng = datagen.rng_for(seed)
    sch = datagen.star_schema(rng, r_T, 3, [(5, 4, "uniform"), (7, 2, "uniform")])
    if positive:
        for s in sch.sources:
            s.D[...] = np.abs(s.D) + 0.5
    return sch


def test_row_and_column_sums_equal_sums_of_the_dense_definition():
    for seed in (41, 42):
        sch = datagen.tiny_random_schema(seed, r_T=11, c_T=6, n=3)
        T = oracle.brute_force_target(sch)
        np.testing.assert_allclose(oracle.row_sum(sch), T.sum(axis=1), rtol=0, atol=1e-6)
        np.testing.assert_allclose(oracle.col_sum(sch), T.sum(axis=0), rtol=0, atol=1e-6)
    sch = _star(43)
    # a star join: colSum = [colSum(S) | fan-out-weighted colSum(R_k)]; every key of R_1 used k_j times
    fk = sch.sources[1].row_idx
    want = np.bincount(fk, minlength=5) @ sch.sources[1].D.astype(np.float64)
    np.testing.assert_allclose(oracle.col_sum(sch)[3:7], want, rtol=1e-6)
    np.testing.assert_allclose(oracle.row_sum(sch).sum(), oracle.col_sum(sch).sum(), rtol=1e-12)


@pytest.mark.parametrize("op,x", [("mul", -1.75), ("div", 3.0), ("add", 0.5), ("sub", 2.0), ("pow", 3.0),
                                  ("exp", 0.0), ("abs", 0.0), ("square", 0.0)])
def test_elementwise_on_the_table_equals_elementwise_on_the_sources_when_every_cell_has_one_feeder(op, x):
    # the claim behind Tab. 2's cost sum_k m_k: with exactly one source cell per target cell the operator can
    # be applied to the source tables and the result assembled afterwards (dense Def. 1 / Def. 2 matrices)
    sch = _star(44)
    assert np.all(oracle.cover_counts(sch) == 1)
    want = oracle.apply_elementwise(oracle.brute_force_target(sch), op, x)
    got = _assemble_dense(sch, [oracle.apply_elementwise(s.D, op, x) for s in sch.sources])
    np.testing.assert_allclose(oracle.elementwise(sch, op, x), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("op", ["log", "sqrt"])
def test_elementwise_functions_with_a_restricted_domain(op):
    sch = _star(45, positive=True)
    want = oracle.apply_elementwise(oracle.brute_force_target(sch), op)
    got = _assemble_dense(sch, [oracle.apply_elementwise(s.D, op) for s in sch.sources])
    np.testing.assert_allclose(oracle.elementwise(sch, op), want, rtol=1e-12)
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_abs_against_a_table_written_by_hand():
    # |t| cell by cell on a table with negative, zero and positive cells; the expected values are typed in
    A = np.array([[-1.5, 2.0, 0.0], [3.25, -0.125, -7.0]])
    want = np.array([[1.5, 2.0, 0.0], [3.25, 0.125, 7.0]])
    assert np.array_equal(oracle.apply_elementwise(A, "abs"), want)
    assert not np.array_equal(oracle.apply_elementwise(A, "abs"), A)
    # on a factorized table: S = [[-1], [2]], R = [[-3, 4]], both target rows join R's only row
    S = np.array([[-1.0], [2.0]], dtype=np.float32)
    R = np.array([[-3.0, 4.0]], dtype=np.float32)
    sch = datagen.Schema([datagen.Source(S, None, np.array([0], dtype=np.int32)),
                          datagen.Source(R, np.array([0, 0], dtype=np.int32), np.array([1, 2], dtype=np.int32))], 2, 3)
    assert np.array_equal(oracle.elementwise(sch, "abs"), np.array([[1.0, 3.0, 4.0], [2.0, 3.0, 4.0]]))


def test_elementwise_closed_forms():
    sch = _star(46, positive=True)
    T = oracle.brute_force_target(sch)
    np.testing.assert_allclose(oracle.apply_elementwise(oracle.elementwise(sch, "log"), "exp"), T, rtol=1e-12)
    np.testing.assert_allclose(oracle.apply_elementwise(oracle.elementwise(sch, "square"), "sqrt"), T, rtol=1e-12)
    np.testing.assert_allclose(oracle.elementwise(sch, "pow", 2.0), oracle.elementwise(sch, "square"), rtol=1e-12)
    np.testing.assert_allclose(oracle.elementwise(sch, "div", 4.0), oracle.elementwise(sch, "mul", 0.25), rtol=1e-12)
    np.testing.assert_allclose(oracle.elementwise(sch, "sub", 1.5), oracle.elementwise(sch, "add", -1.5), rtol=1e-12)
    assert oracle.elementwise(sch, "exp")[0, 0] == pytest.approx(np.exp(float(T[0, 0])), rel=1e-12)


def test_times_and_divide_distribute_over_shared_cells_but_plus_does_not():
    # shared columns and unmatched rows: the product with a scalar is linear, so it may still be applied to the
    # sources; plus is not (a cell with two feeders would receive x twice, an empty cell none)
    sch = datagen.tiny_random_schema(47, r_T=13, c_T=5, n=3)
    C = oracle.cover_counts(sch)
    assert C.max() > 1 and C.min() == 0
    T = oracle.brute_force_target(sch)
    for op, x in (("mul", 2.5), ("div", -4.0)):
        got = _assemble_dense(sch, [oracle.apply_elementwise(s.D, op, x) for s in sch.sources])
        np.testing.assert_allclose(got, oracle.apply_elementwise(T, op, x), rtol=1e-12, atol=1e-12)
    got = _assemble_dense(sch, [oracle.apply_elementwise(s.D, "add", 1.0) for s in sch.sources])
    np.testing.assert_allclose(got, T + C, rtol=1e-12, atol=1e-12)      # x arrives once per feeder
    assert not np.allclose(got, T + 1.0)


def test_cover_counts_from_the_dense_definition():
    sch = datagen.tiny_random_schema(48, r_T=9, c_T=7, n=4)
    want = np.zeros((sch.r_T, sch.c_T))
    for s in sch.sources:
        I = oracle.dense_indicator(s.row_idx, sch.r_T, s.D.shape[0])
        M = oracle.dense_mapping(s.col_map, sch.c_T)
        want += I @ np.ones(s.D.shape) @ M.T
    assert np.array_equal(oracle.cover_counts(sch), want.astype(np.int64))


# ----------------------------------------------------------------------------- cost analysis (Sec. 3)
def test_complexity_of_linear_regression_by_hand_and_by_parts():
    # S 6 x 2 and R 3 x 4 joined into T 6 x 6, written out term by term from Sec. 3.1:
    #   O_mat  = (1*36 + 6*6) + (36 + 6*6)                                  = 144
    #   O_fact = (1*12 + 6*6) + (1*12 + 3*6) + (12 + 2*6) + (12 + 4*6)      = 138
    rng = datagen.rng_for(51)
    sch = datagen.star_schema(rng, 6, 2, [(3, 4, "uniform")])
    assert oracle.complexity_lr(sch) == (144, 138)
    # the T w half is Tab. 2's row for T X with a one-column operand
    mat_lmm, fact_lmm = oracle.complexity_lmm(sch, 1)
    o_mat, o_fact = oracle.complexity_lr(sch)
    assert o_mat - mat_lmm == 6 * 6 + 6 * 6
    assert o_fact - fact_lmm == (12 + 2 * 6) + (12 + 4 * 6)
    # a table that is its own only source has nothing to gain: ratio exactly one
    one = datagen.Schema([datagen.Source(sch.sources[0].D, None, np.arange(2, dtype=np.int32))], 6, 2)
    assert oracle.complexity_lr(one)[0] == oracle.complexity_lr(one)[1]
    assert oracle.tuple_and_feature_ratio(sch) == (2.0, 2.0)


def test_tuple_ratio_and_feature_ratio_on_schemas_where_they_differ():
    # worked by hand (the redundancy measures Sec. 4.3 compares with; config 1 is quoted as "tuple ratio 10 and
    # feature ratio 10" for S 1,000,000 x 20 and R 100,000 x 200, which fixes which ratio is which):
    #   S 6 x 2 joined with R 3 x 8:   tuple ratio = 6 / 3 = 2,     feature ratio = 8 / 2 = 4
    sch = datagen.star_schema(datagen.rng_for(53), 6, 2, [(3, 8, "uniform")])
    assert oracle.tuple_and_feature_ratio(sch) == (2.0, 4.0)
    #   S 20 x 4 joined with R 2 x 2:  tuple ratio = 20 / 2 = 10,   feature ratio = 2 / 4 = 0.5
    sch = datagen.star_schema(datagen.rng_for(54), 20, 4, [(2, 2, "uniform")])
    assert oracle.tuple_and_feature_ratio(sch) == (10.0, 0.5)
    #   two joined tables, S 12 x 3 with R1 4 x 5 and R2 2 x 1:  12 / (4 + 2) = 2,  (5 + 1) / 3 = 2
    #   (and with R2 2 x 4 instead: 2 and 3)
    sch = datagen.star_schema(datagen.rng_for(55), 12, 3, [(4, 5, "uniform"), (2, 4, "uniform")])
    assert oracle.tuple_and_feature_ratio(sch) == (2.0, 3.0)
    # the scaled-down shape of config 1's centre: both ratios 10, neither confused with r_T or c_T
    sch = datagen.star_schema(datagen.rng_for(56), 1_000, 20, [(100, 200, "uniform")])
    assert oracle.tuple_and_feature_ratio(sch) == (10.0, 10.0)


def test_complexity_ratio_grows_with_redundancy():
    # more target rows per dimension row, or wider dimension tables, favour the factorized form (Sec. 3.1)
    def ratio(r_R, c_R):
        sch = datagen.star_schema(datagen.rng_for(52), 1_000, 4, [(r_R, c_R, "uniform")])
        o_mat, o_fact = oracle.complexity_lr(sch)
        return o_mat / o_fact
    assert ratio(10, 8) > ratio(100, 8) > ratio(500, 8)
    assert ratio(100, 40) > ratio(100, 8) > ratio(100, 2)


# ----------------------------------------------------------------------------- right multiply (Tab. 2, row XT)
def test_rmm_equals_dense_definition_and_transposed_tmm():
    for seed in (61, 62):
        sch = datagen.tiny_random_schema(seed, r_T=12, c_T=5, n=3)
        T = oracle.brute_force_target(sch)
        X = datagen.rng_for(seed + 100).standard_normal((4, 12))
        np.testing.assert_allclose(oracle.rmm(sch, X), X @ T, rtol=1e-6, atol=1e-6)
        np.testing.assert_allclose(oracle.rmm(sch, X), oracle.tmm(sch, X.T).T, rtol=1e-12, atol=1e-12)
    # unit vectors pick rows of the table; a row of ones gives colSum
    sch = datagen.tiny_random_schema(63, r_T=7, c_T=4, n=2)
    E = np.eye(7)
    np.testing.assert_allclose(oracle.rmm(sch, E), oracle.Target(sch).T32.astype(np.float64), rtol=0, atol=0)
    np.testing.assert_allclose(oracle.rmm(sch, np.ones((1, 7)))[0], oracle.col_sum(sch), rtol=1e-12)


def test_rmm_complexity_by_hand():
    # S 6 x 2, R 3 x 4, T 6 x 6, X 5 x 6: materialized 5*36 + 6*30 = 360; factorized (5*12 + 2*30) + (5*12 + 4*30) = 300
    sch = datagen.star_schema(datagen.rng_for(64), 6, 2, [(3, 4, "uniform")])
    assert oracle.complexity_rmm(sch, 5) == (360, 300)


# ------------------------------------------------------------------ KMeans (Lloyd iteration)
def _blob_target(rng, n_per, centres, spread):
    """Rows drawn around given centres (in order: n_per rows per centre); returns the target and the labels."""
    k, c = centres.shape
    rows = np.concatenate([centres[j] + spread * rng.standard_normal((n_per, c)) for j in range(k)]).astype(np.float32)
    labels = np.repeat(np.arange(k), n_per)
    order = rng.permutation(rows.shape[0])
    return oracle.Target(table=rows[order]), labels[order]


def test_kmeans_step_equals_a_loop_over_points_and_centroids():
    sch = datagen.tiny_random_schema(31, r_T=23, c_T=5, n=3)
    T = oracle.materialize(sch).astype(np.float64)           # the float32 table (pinned above), widened
    rng = datagen.rng_for(310)
    C = rng.standard_normal((5, 4))
    want_assign, sums, cnt, inertia = [], [[0.0] * 5 for _ in range(4)], [0] * 4, 0.0
    for i in range(23):
        best, best_d = -1, None
        for j in range(4):
            d = sum((T[i][t] - C[t][j]) ** 2 for t in range(5))
            if best_d is None or d < best_d:
                best, best_d = j, d
        want_assign.append(best)
        cnt[best] += 1
        inertia += best_d
        for t in range(5):
            sums[best][t] += T[i][t]
    C_new, assign, counts, got_inertia = oracle.kmeans_step(oracle.Target(sch), C)
    assert list(assign) == want_assign and list(counts) == cnt
    for j in range(4):
        for t in range(5):
            want = sums[j][t] / cnt[j] if cnt[j] else C[t][j]
            assert abs(C_new[t, j] - want) < 1e-12
    assert abs(got_inertia - inertia) < 1e-9


def test_kmeans_step_equals_scipy_vq_and_one_kmeans2_iteration():
    from scipy.cluster.vq import kmeans2, vq
    sch = datagen.config0(seed=5, r_S=3_000, r_R=300)
    tg = oracle.Target(sch)
    rng = datagen.rng_for(311)
    C0 = tg.T32[rng.choice(tg.r_T, 7, replace=False)].astype(np.float64).T          # c_T x 7
    C_new, assign, counts, inertia = oracle.kmeans_step(tg, C0)
    labels, dist = vq(tg.T32.astype(np.float64), C0.T.copy())
    assert np.array_equal(assign, labels)
    np.testing.assert_allclose(inertia, np.sum(dist ** 2), rtol=1e-12)
    centres, labels2 = kmeans2(tg.T32.astype(np.float64), C0.T.copy(), iter=1, minit="matrix")
    assert np.array_equal(assign, labels2)
    np.testing.assert_allclose(C_new, centres.T, rtol=1e-12, atol=1e-12)


def test_kmeans_step_on_separated_blobs_returns_the_group_means_and_keeps_empty_clusters():
    rng = datagen.rng_for(312)
    centres = 50.0 * np.eye(4, 6)
    tg, labels = _blob_target(rng, 200, centres, 0.5)
    start = np.concatenate([centres + 1.0, np.full((1, 6), 1e3)]).T                  # a fifth centroid far away
    C_new, assign, counts, _ = oracle.kmeans_step(tg, start)
    assert np.array_equal(assign, labels) and list(counts) == [200, 200, 200, 200, 0]
    for j in range(4):
        np.testing.assert_allclose(C_new[:, j], tg.T32[labels == j].astype(np.float64).mean(axis=0), rtol=1e-13)
    assert np.array_equal(C_new[:, 4], start[:, 4])
    # at the group means a further step changes nothing
    C_again, assign2, _, _ = oracle.kmeans_step(tg, C_new)
    assert np.array_equal(assign2, labels)
    np.testing.assert_allclose(C_again, C_new, rtol=1e-13)


def test_kmeans_objective_never_increases_and_ties_go_to_the_first_centroid():
    sch = datagen.config0(seed=6, r_S=2_000, r_R=100)
    tg = oracle.Target(sch)
    C = tg.T32[:5].astype(np.float64).T
    last = np.inf
    for _ in range(8):
        C, _, _, inertia = oracle.kmeans_step(tg, C)
        assert inertia <= last * (1 + 1e-12)
        last = inertia
    # two identical centroids: nobody chooses the second
    dup = np.concatenate([C[:, :1], C[:, :1], C[:, 1:]], axis=1)
    _, assign, counts, _ = oracle.kmeans_step(tg, dup)
    assert counts[1] == 0 and not np.any(assign == 1)


def test_kmeans_distances_expand_into_norms_and_a_left_multiply():
    # |t - c|^2 = |t|^2 - 2 t.c + |c|^2 : the form that turns the assignment into T C
    sch = datagen.tiny_random_schema(33, r_T=40, c_T=6, n=3)
    tg = oracle.Target(sch)
    C = datagen.rng_for(313).standard_normal((6, 3))
    T = tg.T32.astype(np.float64)
    want = (T ** 2).sum(axis=1)[:, None] - 2.0 * oracle.lmm(tg, C) + (C ** 2).sum(axis=0)[None, :]
    np.testing.assert_allclose(oracle.kmeans_distances(tg, C), want, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ Gaussian NMF (multiplicative updates)
def _nonneg_target(seed, r_T=300, c_T=12):
    rng = datagen.rng_for(seed)
    return oracle.Target(table=np.abs(rng.standard_normal((r_T, c_T))).astype(np.float32)), rng


def test_gnmf_step_equals_one_iteration_of_sklearn_multiplicative_update():
    import warnings
    from sklearn.decomposition import NMF
    tg, rng = _nonneg_target(320)
    W0, H0 = rng.random((tg.r_T, 4)) + 0.1, rng.random((4, tg.c_T)) + 0.1
    model = NMF(n_components=4, init="custom", solver="mu", beta_loss="frobenius", max_iter=1, tol=0.0)
    with warnings.catch_warnings():
        warnings.simplefilter("ignore")
        W_lib = model.fit_transform(tg.T32.astype(np.float64), W=W0.copy(), H=H0.copy())
    W1, H1 = oracle.gnmf_step(tg, W0, H0)
    np.testing.assert_allclose(W1, W_lib, rtol=1e-12)
    np.testing.assert_allclose(H1, model.components_, rtol=1e-12)


def test_gnmf_step_element_by_element():
    tg, rng = _nonneg_target(321, r_T=7, c_T=5)
    T = tg.T32.astype(np.float64)
    W, H = rng.random((7, 2)) + 0.1, rng.random((2, 5)) + 0.1
    W1 = np.empty_like(W)
    for i in range(7):
        for a in range(2):
            num = sum(T[i, t] * H[a, t] for t in range(5))
            den = sum(W[i, b] * sum(H[b, t] * H[a, t] for t in range(5)) for b in range(2))
            W1[i, a] = W[i, a] * num / den
    H1 = np.empty_like(H)
    for a in range(2):
        for t in range(5):
            num = sum(W1[i, a] * T[i, t] for i in range(7))
            den = sum(sum(W1[i, a] * W1[i, b] for i in range(7)) * H[b, t] for b in range(2))
            H1[a, t] = H[a, t] * num / den
    got_W, got_H = oracle.gnmf_step(tg, W, H)
    np.testing.assert_allclose(got_W, W1, rtol=1e-12)
    np.testing.assert_allclose(got_H, H1, rtol=1e-12)


def test_gnmf_exact_factorization_is_a_fixed_point():
    rng = datagen.rng_for(322)
    W = rng.integers(1, 5, (60, 3)).astype(np.float64)
    H = rng.integers(1, 5, (3, 9)).astype(np.float64)
    tg = oracle.Target(table=(W @ H).astype(np.float32))                             # small integers: exact
    W1, H1 = oracle.gnmf_step(tg, W, H)
    np.testing.assert_allclose(W1, W, rtol=1e-13)
    np.testing.assert_allclose(H1, H, rtol=1e-13)
    assert oracle.gnmf_objective(tg, W, H) == 0.0


def test_gnmf_objective_never_increases_and_factors_stay_nonnegative():
    sch = datagen.config0(seed=7, r_S=1_500, r_R=150)
    for s in sch.sources:
        s.D[...] = np.abs(s.D)
    tg = oracle.Target(sch)
    rng = datagen.rng_for(323)
    W, H = rng.random((tg.r_T, 5)), rng.random((5, tg.c_T))
    last = oracle.gnmf_objective(tg, W, H)
    for _ in range(15):
        W, H = oracle.gnmf_step(tg, W, H)
        now = oracle.gnmf_objective(tg, W, H)
        assert now <= last * (1 + 1e-12) and W.min() >= 0.0 and H.min() >= 0.0
        last = now
    T = tg.T32.astype(np.float64)
    np.testing.assert_allclose(oracle.gnmf_objective(tg, W, H), 0.5 * np.linalg.norm(T - W @ H) ** 2, rtol=1e-12)


def test_gnmf_zero_rows_and_columns_stay_zero_without_dividing_by_zero():
    tg, rng = _nonneg_target(324, r_T=30, c_T=6)
    W, H = rng.random((30, 3)), rng.random((3, 6))
    W[4] = 0.0
    H[:, 2] = 0.0
    W1, H1 = oracle.gnmf_step(tg, W, H)
    assert np.all(np.isfinite(W1)) and np.all(np.isfinite(H1))
    assert np.all(W1[4] == 0.0) and np.all(H1[:, 2] == 0.0)


# ------------------------------------------------------------------ bfloat16-input variant of Alg. 1
def test_round_to_bf16_against_torch_and_hand_values():
    import torch
    rng = datagen.rng_for(321)
    a = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-20, 20, 5000),
                        [0.0, -0.0, 1.0, -1.0, 2.0 ** -126, 3.0e38]]).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_to_bf16(a)
    assert np.array_equal(got, want)
    # 8 significant bits: neighbours of 1 are 1 - 2^-8 and 1 + 2^-7; ties go to the even mantissa
    assert oracle.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0                    # tie, 1.0 is even
    assert oracle.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6    # tie, up to the even one
    assert oracle.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert oracle.round_to_bf16(np.array([1.0 - 2.0 ** -10]))[0] == 1.0
    rel_err = np.abs(got - a.astype(np.float64))[a != 0] / np.abs(a.astype(np.float64))[a != 0]
    assert rel_err.max() <= 2.0 ** -8


def test_gd_bf16_inputs_first_step_is_exact_on_representable_inputs():
    # from w = 0 the first iteration multiplies representable tables by zeros and by -y: no rounding takes place
    rng = datagen.rng_for(322)
    sch = datagen.star_schema(rng, 400, 6, [(30, 5, "uniform")])
    for s in sch.sources:
        s.D[...] = oracle.round_to_bf16(s.D).astype(np.float32)
    tg = oracle.Target(sch)
    y = oracle.round_to_bf16(rng.standard_normal(sch.r_T))
    W1, L1 = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 2)), [0.1, 0.3], 1)
    W2, L2 = oracle.gd_bf16_inputs(tg, "linear", y, np.zeros((sch.c_T, 2)), [0.1, 0.3], 1)
    np.testing.assert_allclose(W2, W1, rtol=1e-13, atol=0)
    np.testing.assert_allclose(L2, L1, rtol=1e-13)
    # a second iteration multiplies by weights that are no bfloat16 numbers: the two differ, by no more than a few u
    W1, _ = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 2)), [0.1, 0.3], 2)
    W2, _ = oracle.gd_bf16_inputs(tg, "linear", y, np.zeros((sch.c_T, 2)), [0.1, 0.3], 2)
    d = np.linalg.norm(W2 - W1) / np.linalg.norm(W1)
    assert 1e-6 < d < 2.0 ** -6


@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("shape", [(5_003, 20, 501, 24, "uniform", 8, 5e-2), (5_003, 3, 200, 24, "uniform", 8, 5e-2),
                                   (5_003, 64, 16, 24, "uniform", 8, 5e-2), (5_003, 50, 333, 24, ("zipf", 1.05), 8, 5e-2),
                                   (20_000, 20, 2_000, 200, "uniform", 20, 1.0), (20_000, 20, 2_000, 200, "uniform", 50, 0.7)])
def test_bf16_gd_weight_tolerance_holds_for_the_emulated_arithmetic(model, shape):
    # the derived bound (tests/tolerances.py) against Alg. 1 with rounded product inputs and exact accumulation,
    # on the kinds of schema the device tests of the reduced-precision variant use; the rounding is visible
    # (error above a hundredth of the bound) and within it
    from tolerances import bf16_gd_weight_tol, lambda_max
    r_S, c_S, r_R, c_R, keys, iters, lr_hi = shape
    rng = datagen.rng_for(323 + c_S + iters)
    sch = datagen.star_schema(rng, r_S, c_S, [(r_R, c_R, keys)])
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(sch.r_T))
    lam = lambda_max(oracle.crossprod(tg), sch.r_T)
    lrs = np.geomspace(1e-3, lr_hi, 6)
    if lrs[-1] * lam >= 1.9:
        lrs = lrs * (1.9 / (lrs[-1] * lam))
    W, _ = oracle.gd(tg, model, y, np.zeros((sch.c_T, len(lrs))), lrs, iters)
    Wb, _ = oracle.gd_bf16_inputs(tg, model, y, np.zeros((sch.c_T, len(lrs))), lrs, iters)
    for j, lr in enumerate(lrs):
        err = np.linalg.norm(Wb[:, j] - W[:, j]) / np.linalg.norm(W[:, j])
        tol = bf16_gd_weight_tol(iters, sch.c_T, sch.r_T, lr, lam)
        assert tol / 100 < err < tol, (j, lr, err, tol)
