"""Device library against the CPU oracle, element by element, on the same seeded inputs.

Sizes here are the ones the oracle finishes in seconds; they span many workgroup tiles, ragged
tails, long and empty inverse-index segments.  Tolerances are the ones the task fixes: bit-exact
for integer work and the join-gather, 1e-5 relative Frobenius error for float32 operators, 1e-4
relative 2-norm for gradient-descent weights.
"""
import ctypes

import numpy as np
import pytest

import datagen
import oracle
from tolerances import bf16_gd_weight_tol, lambda_max

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

OP_TOL = 1e-5
GD_TOL = 1e-4


@pytest.fixture(scope="module")
def il():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_01985_amd as mod
    return mod


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (nb if nb > 0 else 1.0))


def assert_each_element(got, want, A, B, tol=OP_TOL):
    """Per-element bound beside the norm: every entry of a product A @ B computed in float32 lies within
    tol * (|A| @ |B|) of the exact one (the componentwise rounding bound of a sum of products, whatever the
    order of the additions), so no single wrong entry can hide behind the norm of the others."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    scale = np.abs(np.asarray(A, dtype=np.float64)) @ np.abs(np.asarray(B, dtype=np.float64))
    excess = np.abs(got - want) - (tol * scale + 1e-30)
    worst = np.unravel_index(np.argmax(excess), excess.shape) if excess.size else None
    assert excess.size == 0 or excess.max() <= 0, f"entry {worst}: got {got[worst]}, want {want[worst]}, scale {scale[worst]}"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


SCHEMAS = {
    "config0": lambda: datagen.config0(),
    "config1_small": lambda: datagen.config1(r_S=30_011, r_R=3_001, c_R=200),
    "config1_fr1": lambda: datagen.config1(r_S=20_000, r_R=10_000, c_R=20),
    "config1_wide_dim": lambda: datagen.config1(r_S=20_003, r_R=257, c_R=800),
    "config2_small": lambda: datagen.config2(r_S=200_003, dim_rows=(4_000, 2_000, 400)),
    "config3_small": lambda: datagen.config3(rows=50_001, cols=64, shared=32),
    "tiny3": lambda: datagen.tiny_random_schema(3, r_T=9, c_T=7, n=3),
    "tiny_mixed": lambda: datagen.tiny_random_schema(21, r_T=333, c_T=19, n=5),
    "odd_cols": lambda: datagen.star_schema(datagen.rng_for(77), 5_001, 7, [(97, 13, "uniform"), (31, 2, "uniform")]),
}

_cache = {}


def get(il, name, max_cx=17):
    key = (name, max_cx)
    if key not in _cache:
        sch = SCHEMAS[name]()
        tg = oracle.Target(sch)
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=max_cx)
        _cache[key] = (sch, tg, plan)
    return _cache[key]


ALL = list(SCHEMAS)


def _labels(sch, tg, kind):
    return datagen.finish_labels(kind, oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])


# ------------------------------------------------------------------ plan: inverse index (integer, exact)
@pytest.mark.parametrize("name", ["config0", "config2_small", "config3_small", "tiny_mixed"])
def test_inverse_index_exact(il, name):
    sch, tg, plan = get(il, name)
    for k, s in enumerate(sch.sources):
        rowptr, perm = il.ilargi_plan_inverse_index(plan, k)
        if s.row_idx is None:
            assert rowptr is None
            continue
        ident = np.array_equal(s.row_idx[:s.rows], np.arange(s.rows)) and np.all(s.row_idx[s.rows:] == -1)
        if ident:
            assert rowptr is None
            continue
        valid = np.flatnonzero(s.row_idx >= 0)
        want_perm = valid[np.argsort(s.row_idx[valid], kind="stable")].astype(np.int32)
        want_ptr = np.zeros(s.rows + 1, dtype=np.int32)
        want_ptr[1:] = np.cumsum(np.bincount(s.row_idx[valid], minlength=s.rows))
        assert np.array_equal(rowptr, want_ptr)
        assert np.array_equal(perm, want_perm)


def test_inverse_index_matches_oracle_definition(il):
    sch, tg, plan = get(il, "tiny_mixed")
    for k, s in enumerate(sch.sources):
        rowptr, perm = il.ilargi_plan_inverse_index(plan, k)
        if rowptr is None:
            continue
        o_ptr, o_perm, _ = oracle.inverse_index(s.row_idx, s.rows)
        assert np.array_equal(rowptr, o_ptr) and np.array_equal(perm, o_perm)


def test_inverse_index_skewed_and_empty_segments(il):
    rng = datagen.rng_for(5)
    r_T, r_k = 100_000, 5_000
    idx = datagen.bounded_zipf_keys(rng, r_T, r_k, 1.3)
    idx[rng.random(r_T) < 0.1] = -1
    D = rng.standard_normal((r_k, 4)).astype(np.float32)
    sch = datagen.Schema([datagen.Source(D, idx, np.arange(4, dtype=np.int32))], r_T, 4)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, 4, max_cx=3)
    rowptr, perm = il.ilargi_plan_inverse_index(plan, 0)
    valid = np.flatnonzero(idx >= 0)
    cnt = np.bincount(idx[valid], minlength=r_k)
    assert cnt.max() > 2048 * 3 and (cnt == 0).sum() > 0      # long segments and empty ones both occur
    assert np.array_equal(np.diff(rowptr), cnt)
    assert np.array_equal(perm, valid[np.argsort(idx[valid], kind="stable")])
    Y = rng.standard_normal((r_T, 3)).astype(np.float32)
    Z = il.ilargi_segment_sum(plan, 0, dev(Y)).cpu().numpy()
    assert rel(Z, oracle.segment_sum(idx, r_k, Y)) < OP_TOL
    assert np.all(Z[cnt == 0] == 0.0)


# ------------------------------------------------------------------ materialize (bit-exact)
@pytest.mark.parametrize("name", ALL)
def test_materialize_bit_exact(il, name):
    sch, tg, plan = get(il, name)
    T = il.ilargi_materialize(plan).cpu().numpy()
    assert T.shape == tg.T32.shape
    assert np.array_equal(T.view(np.uint32), tg.T32.view(np.uint32))


# ------------------------------------------------------------------ LMM
@pytest.mark.parametrize("name", ALL)
@pytest.mark.parametrize("cx", [1, 2, 3, 4, 5, 16, 17])
def test_lmm(il, name, cx):
    sch, tg, plan = get(il, name)
    X = datagen.rng_for(1000 + cx).standard_normal((sch.c_T, cx)).astype(np.float32)
    got = il.ilargi_lmm(plan, dev(X)).cpu().numpy()
    want = oracle.lmm(tg, X)
    assert rel(got, want) < OP_TOL
    assert_each_element(got, want, tg.T32, X)


@pytest.mark.parametrize("name", ["config0", "tiny_mixed", "odd_cols"])
def test_lmm_identity_operand_reproduces_table(il, name):
    sch, tg, plan = get(il, name, max_cx=32)
    if sch.c_T > 32:
        pytest.skip("operand wider than the plan")
    got = il.ilargi_lmm(plan, dev(np.eye(sch.c_T, dtype=np.float32))).cpu().numpy()
    # every output is 1.0 * cell plus zeros: exact unless two sources share the cell
    np.testing.assert_allclose(got, tg.T32, rtol=1e-6, atol=1e-6)
    if name != "tiny_mixed":
        assert np.array_equal(got, tg.T32)


# ------------------------------------------------------------------ TMM
@pytest.mark.parametrize("name", ALL)
@pytest.mark.parametrize("cx", [1, 2, 3, 4, 5, 8, 13, 16, 17])
def test_tmm(il, name, cx):
    sch, tg, plan = get(il, name)
    Y = datagen.rng_for(2000 + cx).standard_normal((sch.r_T, cx)).astype(np.float32)
    got = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
    want = oracle.tmm(tg, Y)
    assert rel(got, want) < OP_TOL
    assert_each_element(got, want, tg.T32.T, Y)


@pytest.mark.parametrize("name", ["config2_small", "config3_small"])
def test_adjoint_identity_on_device(il, name):
    sch, tg, plan = get(il, name)
    rng = datagen.rng_for(31)
    X = rng.standard_normal((sch.c_T, 4)).astype(np.float32)
    Y = rng.standard_normal((sch.r_T, 4)).astype(np.float32)
    TX = il.ilargi_lmm(plan, dev(X)).cpu().numpy().astype(np.float64)
    TtY = il.ilargi_tmm(plan, dev(Y)).cpu().numpy().astype(np.float64)
    lhs, rhs = np.sum(TX * Y), np.sum(X * TtY)
    assert abs(lhs - rhs) < 1e-5 * np.sqrt(np.sum(TX ** 2) * np.sum(Y.astype(np.float64) ** 2))


@pytest.mark.parametrize("name", ["config2_small", "config3_small", "tiny_mixed"])
@pytest.mark.parametrize("cx", [1, 4, 16])
def test_segment_sum(il, name, cx):
    sch, tg, plan = get(il, name)
    Y = datagen.rng_for(3000 + cx).standard_normal((sch.r_T, cx)).astype(np.float32)
    for k, s in enumerate(sch.sources):
        if s.row_idx is None:
            continue
        Z = il.ilargi_segment_sum(plan, k, dev(Y)).cpu().numpy()
        want = np.zeros((s.rows, cx))
        ok = s.row_idx >= 0
        np.add.at(want, s.row_idx[ok], Y[ok].astype(np.float64))
        assert rel(Z, want) < OP_TOL


# ------------------------------------------------------------------ wide operands (matrix-core kernels)
@pytest.mark.parametrize("cx", [8, 12, 16])
@pytest.mark.parametrize("c_S", [4, 8, 12, 20, 28, 44, 64])
def test_transposed_multiply_of_a_short_row_entity_table(il, c_S, cx):
    # the flat-stream column reduce: 1..16 float4 per row (64 / nvec whole rows per wavefront step, with idle lanes
    # when nvec does not divide 64), a row count that ends inside a step, rows beyond the entity table
    rng = datagen.rng_for(5300 + c_S + cx)
    r_S, extra, r_R, c_R = 3_011, 7, 97, 12
    r_T = r_S + extra                                        # the last target rows have no entity row
    S = rng.standard_normal((r_S, c_S)).astype(np.float32)
    R = rng.standard_normal((r_R, c_R)).astype(np.float32)
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    idx_S = np.concatenate([np.arange(r_S), np.full(extra, -1)]).astype(np.int32)
    c_T = c_S + c_R
    sch = datagen.Schema([datagen.Source(S, idx_S, np.arange(c_S, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(c_S, c_T, dtype=np.int32))], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=16)
    Y = rng.standard_normal((r_T, cx)).astype(np.float32)
    G1 = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
    assert rel(G1, oracle.tmm(tg, Y)) < OP_TOL
    assert np.array_equal(G1, il.ilargi_tmm(plan, dev(Y)).cpu().numpy())


@pytest.mark.parametrize("cx", [8, 12, 16])
@pytest.mark.parametrize("c_S,r_R,c_R", [(20, 1_001, 36), (64, 517, 208), (4, 2_000, 100), (12, 8_000, 64)])
def test_transposed_multiply_with_the_flat_reduce_and_the_join_order_pass_in_one_launch(il, c_S, r_R, c_R, cx):
    # identity source with short rows + joined source, operands of whole float4 rows: both parts share a launch
    # (roles dealt to groups of eight workgroups).  Ragged row tiles on both sides, 3 / 13 / 7 / 4 column tiles of
    # the joined table, keys that are missing (-1), rows of the joined table nobody joins (r_R = 8000 > r_T), a
    # third source whose join-order pass runs in a launch of its own; results repeat bit for bit
    rng = datagen.rng_for(5300 + c_S + cx)
    r_T, r_Q, c_Q = 7_003, 701, 24
    S = rng.standard_normal((r_T, c_S)).astype(np.float32)
    R = rng.standard_normal((r_R, c_R)).astype(np.float32)
    Q = rng.standard_normal((r_Q, c_Q)).astype(np.float32)
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    fk[::23] = -1
    fq = rng.integers(0, r_Q, r_T).astype(np.int32)
    c_T = c_S + c_R + c_Q
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c_S, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(c_S, c_S + c_R, dtype=np.int32)),
                          datagen.Source(Q, fq, np.arange(c_S + c_R, c_T, dtype=np.int32))], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=16)
    Y = rng.standard_normal((r_T, cx)).astype(np.float32)
    il.ilargi_plan_trace_begin(plan, "*", 16)
    G1 = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
    _, names = il.ilargi_plan_trace_end(plan, 16, names=True)
    assert any(n.startswith("colred+join") for n in names), names
    want = oracle.tmm(tg, Y)
    assert rel(G1, want) < OP_TOL
    assert_each_element(G1, want, tg.T32.T, Y)
    assert np.array_equal(G1, il.ilargi_tmm(plan, dev(Y)).cpu().numpy())


@pytest.mark.parametrize("cx", [8, 13, 17, 32])
@pytest.mark.parametrize("c_R", [64, 100, 260, 516])
def test_transposed_multiply_of_a_wide_joined_table_with_few_operand_columns(il, c_R, cx):
    # the column-split reduction: table widths that end inside a 64-column slab, beyond the four slabs of one
    # workgroup (260, 516 columns), operand widths around the 16-column tiles, few rows per chunk
    rng = datagen.rng_for(5200 + c_R + cx)
    r_T, r_R, c_S = 2_003, 333, 4
    S = rng.standard_normal((r_T, c_S)).astype(np.float32)
    R = rng.standard_normal((r_R, c_R)).astype(np.float32)
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    fk[::19] = -1
    c_T = c_S + c_R
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c_S, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(c_S, c_T, dtype=np.int32))], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=32)
    Y = rng.standard_normal((r_T, cx)).astype(np.float32)
    G1 = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
    assert rel(G1, oracle.tmm(tg, Y)) < OP_TOL
    assert np.array_equal(G1, il.ilargi_tmm(plan, dev(Y)).cpu().numpy())


@pytest.mark.parametrize("cx", [33, 64, 65, 100, 130, 192])
@pytest.mark.parametrize("c_R", [4, 36, 72, 200])
def test_wide_product_of_a_joined_table_chunk_and_slab_tails(il, c_R, cx):
    # the chunked product kernel for 64-column slabs: table widths that end inside a 32-column chunk or a 16-column
    # group, row counts off the 128-row block, operand widths that end inside a slab and are not float4 multiples,
    # unmapped table columns
    rng = datagen.rng_for(5100 + c_R)
    r_T, r_R, c_S = 3_001, 1_157, 8
    S = rng.standard_normal((r_T, c_S)).astype(np.float32)
    R = rng.standard_normal((r_R, c_R)).astype(np.float32)
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    fk[::17] = -1
    cm = np.arange(c_S, c_S + c_R, dtype=np.int32)
    cm[1::5] = -1                                            # every fifth table column feeds nothing
    live = cm[cm >= 0]
    cm[cm >= 0] = c_S + np.arange(live.size, dtype=np.int32)
    c_T = c_S + live.size
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c_S, dtype=np.int32)), datagen.Source(R, fk, cm)], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=192)
    X = rng.standard_normal((c_T, cx)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL



@pytest.mark.parametrize("prec", ["f32", "bf16"])
@pytest.mark.parametrize("r_R,c_R,cx", [(31, 4, 64), (1_157, 20, 100), (5_003, 100, 256), (2_050, 256, 300),
                                        (1_024, 204, 68), (4_097, 36, 64)])
def test_streaming_wide_product_and_column_reduce_tails(il, prec, r_R, c_R, cx):
    # the streaming kernels of the wide batch (operand slab in LDS, table rows straight into the matrix cores; the
    # column reduce with its whole result block in registers): table widths of 1 to 16 column groups and ones that
    # end inside a group or inside a 32-column step, row counts below one tile / one 32-row step and off both,
    # operand widths that end inside a slab or need a second slab, keys missing, unmapped table columns.  Inputs
    # are small integers (exact in bfloat16, sums exact in float32), so both precisions must equal the oracle.
    rng = datagen.rng_for(5200 + c_R + cx)
    r_T, c_S = 6_011, 8
    S = rng.integers(-3, 4, (r_T, c_S)).astype(np.float32)
    R = rng.integers(-3, 4, (r_R, c_R)).astype(np.float32)
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    fk[::13] = -1
    cm = np.arange(c_S, c_S + c_R, dtype=np.int32)
    if c_R > 4:
        cm[2::7] = -1
        live = cm[cm >= 0]
        cm[cm >= 0] = c_S + np.arange(live.size, dtype=np.int32)
        c_T = c_S + live.size
    else:
        c_T = c_S + c_R
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c_S, dtype=np.int32)), datagen.Source(R, fk, cm)], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=cx)
    code = il.F32 if prec == "f32" else il.BF16_IN_F32_ACC
    X = rng.integers(-2, 3, (c_T, cx)).astype(np.float32)
    Y = rng.integers(-2, 3, (r_T, cx)).astype(np.float32)
    got = il.ilargi_lmm(plan, dev(X), precision=code).cpu().numpy()
    assert np.array_equal(got, oracle.lmm(tg, X).astype(np.float32))
    got = il.ilargi_tmm(plan, dev(Y), precision=code).cpu().numpy()
    assert np.array_equal(got, oracle.tmm(tg, Y).astype(np.float32))
    names = _traced_kernels(il, plan, lambda: il.ilargi_lmm(plan, dev(X), precision=code))
    assert any(n.startswith("lmm_rows") for n in names), names


@pytest.mark.parametrize("name", ["config1_small", "config1_wide_dim", "config3_small", "odd_cols", "tiny_mixed"])
@pytest.mark.parametrize("cx", [8, 40, 64, 256])
def test_wide_operands(il, name, cx):
    sch, tg, plan = get(il, name, max_cx=256)
    rng = datagen.rng_for(5000 + cx)
    X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
    Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL


def test_gd_wide_batch_of_models(il):
    # the batched hyper-parameter sweep at reduced size: 64 models, log-spaced learning rates
    sch = datagen.config4(r_S=40_007, r_R=4_001, c_R=200, models=64)
    tg = oracle.Target(sch)
    y = _labels(sch, tg, "linear")
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=64)
    lrs = sch.extras["lr"]
    W, L = _run_gd(il, plan, il.LINEAR, y, lrs, 20, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 64)), lrs, 20)
    errs = [rel(W[:, j], W_ref[:, j]) for j in range(64)]
    assert max(errs) < GD_TOL, max(errs)
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


def test_gd_logistic_wide(il):
    sch, tg, plan = get(il, "config2_small", max_cx=256)
    y = _labels(sch, tg, "logistic")
    lrs = np.linspace(0.05, 0.5, 16)
    W, L = _run_gd(il, plan, il.LOGISTIC, y, lrs, 10, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "logistic", y, np.zeros((sch.c_T, 16)), lrs, 10)
    assert max(rel(W[:, j], W_ref[:, j]) for j in range(16)) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("c_S,m", [(7, 33), (20, 100), (48, 64), (64, 40), (65, 40)])
def test_gd_wide_entity_gradient_in_the_assembly_pass(il, model, c_S, m):
    # batches above 32 models form the entity table's block of T^T E while its rows are staged for T W
    # (tables up to 64 columns; 65 takes the separate reduction); ragged slabs, unaligned rows, both models
    rng = datagen.rng_for(900 + c_S)
    sch = datagen.star_schema(rng, 5_003, c_S, [(301, 24, "uniform"), (57, 9, ("zipf", 1.1))])
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(sch.r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=m)
    lrs = np.geomspace(1e-3, 5e-2, m)
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    W, L = _run_gd(il, plan, code, y, lrs, 8, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, m)), lrs, 8)
    assert max(rel(W[:, j], W_ref[:, j]) for j in range(m)) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


@pytest.mark.parametrize("prec", ["f32", "bf16"])
@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("c_S,r_R,keys,m", [(20, 501, "uniform", 64), (7, 333, ("zipf", 1.05), 33),
                                            (48, 8_000, "uniform", 100), (64, 16, "uniform", 40),
                                            (36, 501, "uniform", 64), (50, 333, ("zipf", 1.05), 40),
                                            (3, 200, "uniform", 33)])
def test_gd_wide_star_join_pass(il, prec, model, c_S, r_R, keys, m):
    # entity table plus one dimension table that every row joins, more than 32 models: the pass in join order
    # (residual never stored); ragged tiles of R, rows of R nobody joins (r_R = 8000 > r_T / 2), skewed keys,
    # unaligned and 64-column entity tables, ragged model slabs; 20, 36, 50 and 3 columns leave 1..4 columns
    # beyond whole groups of 16, which ride in the segment-sum MFMA (12-row tiles of R)
    rng = datagen.rng_for(1000 + c_S)
    sch = datagen.star_schema(rng, 5_003, c_S, [(r_R, 24, keys)])
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(sch.r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=m)
    lrs = np.geomspace(1e-3, 5e-2, m)
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    W = torch.zeros((sch.c_T, m), device="cuda")
    lr = dev(lrs.astype(np.float32)); loss = torch.zeros(m, device="cuda"); yd = dev(y)
    L = []
    for _ in range(8):
        il.ilargi_gd_step(plan, code, W, yd, lr, loss,
                          precision=il.F32 if prec == "f32" else il.BF16_IN_F32_ACC)
        L.append(loss.cpu().numpy().copy())
    W = W.cpu().numpy()
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, m)), lrs, 8)
    if prec == "f32":
        assert max(rel(W[:, j], W_ref[:, j]) for j in range(m)) < GD_TOL
        np.testing.assert_allclose(np.array(L), L_ref, rtol=2e-4)
    else:
        # weights under bfloat16 inputs: the bound derived in tests/tolerances.py, per model
        lam = lambda_max(oracle.crossprod(tg), sch.r_T)
        for j in range(m):
            assert rel(W[:, j], W_ref[:, j]) < bf16_gd_weight_tol(8, sch.c_T, sch.r_T, lrs[j], lam), j
        np.testing.assert_allclose(np.array(L), L_ref, rtol=5e-2, atol=2e-2)


# ------------------------------------------------------------------ bfloat16-input variant
BF16_TOL = 5e-3


def _to_bf16_grid(a):
    """Round float32 values to the nearest bfloat16 (ties to even), kept as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


@pytest.mark.parametrize("name", ["config1_small", "config3_small", "odd_cols"])
@pytest.mark.parametrize("cx", [8, 16, 64, 100])
def test_bf16_inputs_within_bound(il, name, cx):
    sch, tg, plan = get(il, name, max_cx=256)
    rng = datagen.rng_for(7000 + cx)
    X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
    Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
    e1 = rel(il.ilargi_lmm(plan, dev(X), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.lmm(tg, X))
    e2 = rel(il.ilargi_tmm(plan, dev(Y), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.tmm(tg, Y))
    assert e1 < BF16_TOL and e2 < BF16_TOL, (e1, e2)
    # the rounding really happens: the result is not the float32 one
    assert e1 > 1e-5 and e2 > 1e-5


def test_bf16_exact_on_representable_inputs(il):
    # tables and operands that already sit on the bfloat16 grid lose nothing: float32 tolerance applies
    sch = datagen.config1(r_S=20_011, r_R=2_003, c_R=200)
    for s in sch.sources:
        s.D[...] = _to_bf16_grid(s.D)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=64)
    rng = datagen.rng_for(71)
    X = _to_bf16_grid(rng.standard_normal((sch.c_T, 64)).astype(np.float32))
    Y = _to_bf16_grid(rng.standard_normal((sch.r_T, 64)).astype(np.float32))
    assert rel(il.ilargi_lmm(plan, dev(X), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    # T^T Y: the segment sums of Y are rounded again before the product, so only the identity source is exact
    splan = il.ilargi_plan_create(il.schema_to_device(sch)[:1], sch.r_T, 20, max_cx=64)
    tgS = oracle.Target(datagen.Schema(sch.sources[:1], sch.r_T, 20))
    assert rel(il.ilargi_tmm(splan, dev(Y), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.tmm(tgS, Y)) < OP_TOL


def test_bf16_needs_a_wide_operand(il):
    sch, tg, plan = get(il, "config0")
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_lmm(plan, torch.zeros((sch.c_T, 4), device="cuda"), precision=il.BF16_IN_F32_ACC)
    assert ei.value.status == il.ERR_UNSUPPORTED


def test_bf16_gradient_descent_tracks_float32(il):
    # weights under bfloat16 inputs: the bound derived in tests/tolerances.py, per model
    sch = datagen.config4(r_S=40_007, r_R=4_001, c_R=200, models=32)
    tg = oracle.Target(sch)
    y = _labels(sch, tg, "linear")
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=32)
    lrs = sch.extras["lr"]
    m = len(lrs)
    W = torch.zeros((sch.c_T, m), device="cuda")
    lr = dev(lrs.astype(np.float32)); loss = torch.zeros(m, device="cuda"); yd = dev(y)
    for _ in range(20):
        il.ilargi_gd_step(plan, il.LINEAR, W, yd, lr, loss, precision=il.BF16_IN_F32_ACC)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, m)), lrs, 20)
    errs = [rel(W.cpu().numpy()[:, j], W_ref[:, j]) for j in range(m)]
    lam = lambda_max(oracle.crossprod(tg), sch.r_T)
    for j in range(m):
        assert errs[j] < bf16_gd_weight_tol(20, sch.c_T, sch.r_T, lrs[j], lam), (j, errs[j])
    # models that have converged sit on the noise floor the input rounding leaves in the residual
    np.testing.assert_allclose(loss.cpu().numpy(), L_ref[-1], rtol=5e-2, atol=2e-2)


@pytest.mark.parametrize("c_S,m", [(20, 64), (48, 40)])
def test_bf16_first_gradient_step_exact_on_representable_inputs(il, c_S, m):
    # from W = 0 the residual is -y; with tables and labels on the bfloat16 grid the entity table's block of the
    # first step (formed in the assembly pass for more than 32 models) rounds nothing and meets the float32
    # bound; the dimension table's block multiplies segment sums of -y, which do get rounded
    rng = datagen.rng_for(950 + c_S)
    sch = datagen.star_schema(rng, 5_003, c_S, [(301, 24, "uniform")])
    for s in sch.sources:
        s.D[...] = _to_bf16_grid(s.D)
    tg = oracle.Target(sch)
    y = _to_bf16_grid(rng.standard_normal(sch.r_T).astype(np.float32)).astype(np.float64)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=m)
    lrs = np.geomspace(1e-3, 5e-2, m)
    W = torch.zeros((sch.c_T, m), device="cuda")
    loss = torch.zeros(m, device="cuda")
    il.ilargi_gd_step(plan, il.LINEAR, W, dev(y.astype(np.float32)), dev(lrs.astype(np.float32)), loss,
                      precision=il.BF16_IN_F32_ACC)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, m)), lrs, 1)
    W = W.cpu().numpy()
    assert max(rel(W[:c_S, j], W_ref[:c_S, j]) for j in range(m)) < OP_TOL
    assert max(rel(W[c_S:, j], W_ref[c_S:, j]) for j in range(m)) < BF16_TOL
    np.testing.assert_allclose(loss.cpu().numpy(), L_ref[-1], rtol=2e-4)


# ------------------------------------------------------------------ crossprod
@pytest.mark.parametrize("name", ALL)
def test_crossprod(il, name):
    sch, tg, plan = get(il, name)
    G = il.ilargi_crossprod(plan).cpu().numpy()
    want = oracle.crossprod(tg)
    assert rel(G, want) < OP_TOL
    assert_each_element(G, want, tg.T32.T, tg.T32)
    assert np.array_equal(G, G.T)


# ------------------------------------------------------------------ gradient descent (Alg. 1)
def _run_gd(il, plan, model, y, lrs, iters, c_T):
    m = len(lrs)
    W = torch.zeros((c_T, m), device="cuda")
    lr = dev(np.asarray(lrs, dtype=np.float32))
    loss = torch.zeros(m, device="cuda")
    yd = dev(y)
    losses = []
    for _ in range(iters):
        il.ilargi_gd_step(plan, model, W, yd, lr, loss)
        losses.append(loss.cpu().numpy().copy())
    return W.cpu().numpy(), np.array(losses)


def test_gd_linear_config0(il):
    sch, tg, plan = get(il, "config0")
    y = _labels(sch, tg, "linear")
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.1], 20, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.1], 20)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)


def test_gd_logistic_config2(il):
    sch, tg, plan = get(il, "config2_small")
    y = _labels(sch, tg, "logistic")
    W, L = _run_gd(il, plan, il.LOGISTIC, y, [0.5], 50, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "logistic", y, np.zeros((sch.c_T, 1)), [0.5], 50)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    assert abs(L[0, 0] - np.log(2.0)) < 1e-6


def test_gd_linear_config3(il):
    sch, tg, plan = get(il, "config3_small")
    y = _labels(sch, tg, "linear")
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.1], 10, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.1], 10)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)


@pytest.mark.parametrize("m", [3, 8, 17])
def test_gd_many_models_one_learning_rate_each(il, m):
    sch, tg, plan = get(il, "config1_small")
    rng = datagen.rng_for(4)
    w_star = rng.standard_normal(sch.c_T)
    y = datagen.finish_labels("linear", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(sch.r_T))
    lrs = np.logspace(-3, 0, m)
    W, L = _run_gd(il, plan, il.LINEAR, y, lrs, 20, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, m)), lrs, 20)
    errs = [rel(W[:, j], W_ref[:, j]) for j in range(m)]
    assert max(errs) < GD_TOL, errs
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("r_T,c_S,r_R,c_R", [(999, 4, 1000, 8), (16_384, 4, 1_024, 16), (8_192, 8, 300, 4), (5_120, 12, 77, 12),
                                             (4_096, 16, 1, 16), (16_000, 4, 0, 0), (5_000, 12, 0, 0), (3, 16, 2, 4)])
def test_gd_small_star_join_in_one_workgroup(il, model, r_T, c_S, r_R, c_R):
    # schemas small enough for the single-launch iteration: every row length of the two tables (1..4 float4), the
    # largest sizes the path takes, fewer rows than threads, a table alone (no joined source), a one-row table
    rng = datagen.rng_for(7000 + r_T + c_S + c_R)
    dims = [(r_R, c_R, "uniform")] if r_R > 0 else []
    sch = datagen.star_schema(rng, r_T, c_S, dims)
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=3)
    lrs = [0.1, 0.02, 0.3]
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    W, L = _run_gd(il, plan, code, y, lrs, 6, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 3)), lrs, 6)
    assert max(rel(W[:, j], W_ref[:, j]) for j in range(3)) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    W2, L2 = _run_gd(il, plan, code, y, lrs, 6, sch.c_T)
    assert np.array_equal(W, W2) and np.array_equal(L, L2)          # same bits on every run


def test_gd_small_star_join_with_missing_keys_shared_and_unfed_columns(il):
    # the joined table listed first, a target column fed by both tables, one fed by nobody, one source column
    # dropped, target rows without a key, rows of the joined table nobody uses
    rng = datagen.rng_for(7100)
    r_T, r_R = 3_000, 200
    S = rng.standard_normal((r_T, 8)).astype(np.float32)
    R = rng.standard_normal((r_R, 4)).astype(np.float32)
    fk = rng.integers(0, r_R // 2, size=r_T).astype(np.int32)
    fk[rng.random(r_T) < 0.1] = -1
    sch = datagen.Schema([datagen.Source(R, fk, np.array([9, 2, -1, 10], dtype=np.int32)),
                          datagen.Source(S, None, np.array([0, 1, 2, 3, 4, 5, 6, 7], dtype=np.int32))], r_T, 12)
    tg = oracle.Target(sch)
    y = rng.standard_normal(r_T).astype(np.float32)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.2], 8, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.2], 8)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    assert W[8, 0] == 0.0 and W[11, 0] == 0.0                       # columns nobody feeds keep their weight


@pytest.mark.parametrize("c_S", [2, 6, 10, 14, 18])
def test_entity_table_with_8_byte_aligned_rows_read_as_row_pairs(il, c_S):
    # entity tables whose number of columns is 2 modulo 4 (and whose row count is even) are streamed as pairs of
    # rows: left multiply with 1..4 operand columns, gradient descent with the fused gradient block (linear and
    # logistic), several chunks per wavefront, a ragged last chunk, keys missing for some rows
    rng = datagen.rng_for(7200 + c_S)
    r_T = 70_002
    sch = datagen.star_schema(rng, r_T, c_S, [(977, 12, "uniform"), (61, 5, ("zipf", 1.2))])
    sch.sources[1].row_idx[rng.random(r_T) < 0.05] = -1
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=4)
    for cx in (1, 2, 3, 4):
        X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
        got = il.ilargi_lmm(plan, dev(X)).cpu().numpy()
        want = oracle.lmm(tg, X)
        assert rel(got, want) < OP_TOL
        assert_each_element(got, want, tg.T32, X)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    for model, code in (("linear", il.LINEAR), ("logistic", il.LOGISTIC)):
        y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(r_T))
        lrs = [0.1, 0.3]
        W, L = _run_gd(il, plan, code, y, lrs, 5, sch.c_T)
        W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 2)), lrs, 5)
        assert max(rel(W[:, j], W_ref[:, j]) for j in range(2)) < GD_TOL
        np.testing.assert_allclose(L, L_ref, rtol=1e-4)
        W2, _ = _run_gd(il, plan, code, y, lrs, 5, sch.c_T)
        assert np.array_equal(W, W2)


@pytest.mark.parametrize("c_S,ndims", [(4, 1), (8, 2), (12, 3), (16, 1), (20, 1), (24, 2), (32, 3), (6, 3), (10, 3), (14, 1)])
def test_one_operand_column_with_one_lane_per_target_row(il, c_S, ndims):
    # one operand column / one model over an entity table with short rows: with 6, 10 or 14 columns every pair of
    # (8-byte aligned) rows lives in one lane after a transposing pass through LDS; the other row lengths take the
    # flat-stream assembly.  1 .. 8 float4 per row, 3 / 5 / 7 float4 per row pair, one to three gathered tables, keys missing for some rows, several steps per wavefront and a ragged
    # last step (70,002 rows), a table smaller than one step (38 rows); plain product, linear and logistic
    # gradient descent against the oracle; results repeat bit for bit
    rng = datagen.rng_for(7300 + c_S)
    dims = [(977, 12, "uniform"), (61, 5, ("zipf", 1.2)), (3_001, 4, "uniform")][:ndims]
    for r_T in (70_002, 38):
        sch = datagen.star_schema(rng, r_T, c_S, dims)
        sch.sources[1].row_idx[rng.random(r_T) < 0.05] = -1
        tg = oracle.Target(sch)
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
        X = rng.standard_normal((sch.c_T, 1)).astype(np.float32)
        got = il.ilargi_lmm(plan, dev(X)).cpu().numpy()
        want = oracle.lmm(tg, X)
        assert rel(got, want) < OP_TOL
        assert_each_element(got, want, tg.T32, X)
        w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
        for model, code in (("linear", il.LINEAR), ("logistic", il.LOGISTIC)):
            y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(r_T))
            W, L = _run_gd(il, plan, code, y, [0.3], 5, sch.c_T)
            W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 1)), [0.3], 5)
            assert rel(W, W_ref) < GD_TOL
            np.testing.assert_allclose(L, L_ref, rtol=1e-4)
            W2, _ = _run_gd(il, plan, code, y, [0.3], 5, sch.c_T)
            assert np.array_equal(W, W2)


def _traced_kernels(il, plan, call):
    il.ilargi_plan_trace_begin(plan, "*", 64)
    call()
    _, names = il.ilargi_plan_trace_end(plan, 64, names=True)
    return names


@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("rows,cols,shared,overlap", [(20_011, 64, 32, 0.3), (70_001, 36, 4, 0.5), (2_000, 8, 8, 1.0),
                                                      (50_000, 4, 0, 0.0)])
def test_gd_union_of_two_sources_joined_on_the_fly(il, model, rows, cols, shared, overlap):
    # union-style integration (every table row lands on one target row): one model trains in a single pass that
    # reads every table once.  Row lengths of 1 .. 16 float4, shared columns, all / some / no entities matched,
    # several steps per wavefront and a ragged last step.
    sch = datagen.config3(seed=7300 + cols, rows=rows, cols=cols, shared=shared, overlap=overlap)
    tg = oracle.Target(sch)
    rng = datagen.rng_for(7301 + cols)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(sch.r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=2)
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    W, L = _run_gd(il, plan, code, y, [0.2], 6, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 1)), [0.2], 6)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    W2, L2 = _run_gd(il, plan, code, y, [0.2], 6, sch.c_T)
    assert np.array_equal(W, W2) and np.array_equal(L, L2)
    Wd = torch.zeros((sch.c_T, 1), device="cuda")
    names = _traced_kernels(il, plan, lambda: il.ilargi_gd_step(plan, code, Wd, dev(y), dev(np.array([0.2], dtype=np.float32)),
                                                                 torch.zeros(1, device="cuda")))
    assert any(n.startswith("gd_rowjoin") for n in names), names
    # two models at once take the general path and agree with it
    W3, _ = _run_gd(il, plan, code, y, [0.2, 0.2], 6, sch.c_T)
    assert rel(W3[:, 0], W_ref[:, 0]) < GD_TOL and rel(W3[:, 1], W_ref[:, 0]) < GD_TOL


def test_gd_union_of_three_sources_with_missing_rows_and_dropped_columns(il):
    # three tables side by side, none of them an identity source: permuted keys, target rows that some tables do
    # not reach, a table column that feeds no target column, a target column fed by two tables, one fed by nobody
    rng = datagen.rng_for(7400)
    r_T = 40_007
    sources = []
    widths = (12, 64, 20)
    col0 = (0, 10, 74)                                   # columns 10, 11 are shared by the first two tables
    for k, ck in enumerate(widths):
        r_k = r_T - 1000 * k
        D = rng.standard_normal((r_k, ck)).astype(np.float32)
        idx = np.full(r_T, -1, dtype=np.int32)
        where = rng.permutation(r_T)[:r_k - 500]         # 500 rows of every table stay unused
        idx[where] = rng.permutation(r_k)[:r_k - 500].astype(np.int32)
        cm = np.arange(col0[k], col0[k] + ck, dtype=np.int32)
        if k == 2:
            cm[3] = -1
        sources.append(datagen.Source(D, idx, cm))
    c_T = 96                                             # columns 94, 95 fed by nobody
    sch = datagen.Schema(sources, r_T, c_T)
    tg = oracle.Target(sch)
    y = rng.standard_normal(r_T).astype(np.float32)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.1], 5, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.1], 5)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    assert W[94, 0] == 0.0 and W[95, 0] == 0.0 and W[77, 0] == 0.0
    Wd = torch.zeros((sch.c_T, 1), device="cuda")
    names = _traced_kernels(il, plan, lambda: il.ilargi_gd_step(plan, il.LINEAR, Wd, dev(y), dev(np.array([0.1], dtype=np.float32)),
                                                                 torch.zeros(1, device="cuda")))
    assert any(n.startswith("gd_rowjoin") for n in names), names


def test_gd_without_loss_output(il):
    sch, tg, plan = get(il, "config0")
    y = _labels(sch, tg, "linear")
    W = torch.zeros((sch.c_T, 1), device="cuda")
    il.ilargi_gd_step(plan, il.LINEAR, W, dev(y), dev(np.array([0.1], dtype=np.float32)), None)
    W_ref, _ = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.1], 1)
    assert rel(W.cpu().numpy(), W_ref) < GD_TOL


@pytest.mark.parametrize("c_R", [65, 77, 200, 208])
def test_crossprod_symmetric_block_of_a_wide_dimension_table(il, c_R):
    # tables with 65..208 columns take the upper-triangle kernel for their diagonal block; ragged last tile,
    # unaligned rows (77), skewed fan-out as row weights, rows of R that nobody joins
    rng = datagen.rng_for(1100 + c_R)
    sch = datagen.star_schema(rng, 3_001, 5, [(1_237, c_R, ("zipf", 1.1))])
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL
    assert np.array_equal(G, G.T)


@pytest.mark.parametrize("rows,cols,shared,overlap", [(50_001, 64, 32, 0.3), (7_003, 36, 4, 0.5), (12_345, 52, 52, 1.0),
                                                      (9_999, 40, 0, 0.0), (33, 64, 16, 0.4), (20_000, 8, 8, 0.25)])
def test_crossprod_of_stacked_tables_with_at_most_64_columns(il, rows, cols, shared, overlap):
    # union-style integration: the diagonal blocks of tables with 36..64 columns and the block of the row pairs both
    # tables feed run as streaming matrix-core kernels over interleaved column tiles.  Ragged runs (rows that are no
    # multiple of 32), column counts that leave lanes idle (36, 40, 52), every / no / some entities in both tables
    # (no pairs at all: the block is zero), a table of 8 columns (pair block only), fewer rows than one run;
    # symmetric to the bit and the same bits on a second call
    sch = datagen.config3(seed=900 + cols, rows=rows, cols=cols, shared=shared, overlap=overlap)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    G = il.ilargi_crossprod(plan).cpu().numpy()
    want = oracle.crossprod(tg)
    assert rel(G, want) < OP_TOL
    assert_each_element(G, want, tg.T32.T, tg.T32)
    assert np.array_equal(G, G.T)
    assert np.array_equal(G, il.ilargi_crossprod(plan).cpu().numpy())


@pytest.mark.parametrize("c_R", [36, 48, 64])
def test_crossprod_weighted_diagonal_block_of_a_joined_table_with_at_most_64_columns(il, c_R):
    # the fan-out of a joined table's rows weighs its diagonal block: skewed keys, rows nobody joins (weight 0),
    # a second joined table whose pair block with the first goes through the listed row pairs
    rng = datagen.rng_for(1400 + c_R)
    sch = datagen.star_schema(rng, 9_001, 40, [(7_000, c_R, ("zipf", 1.1)), (6_500, 12, "uniform")])
    sch.sources[2].row_idx[rng.random(sch.r_T) < 0.3] = -1
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    G = il.ilargi_crossprod(plan).cpu().numpy()
    want = oracle.crossprod(tg)
    assert rel(G, want) < OP_TOL
    assert_each_element(G, want, tg.T32.T, tg.T32)
    assert np.array_equal(G, G.T)


@pytest.mark.parametrize("c_S,r_R,dist", [(1, 100, "uniform"), (5, 1_237, ("zipf", 1.3)), (16, 999, "uniform"),
                                           (17, 1_601, ("zipf", 1.1)), (20, 2_000, "uniform"), (31, 17, "uniform"),
                                           (32, 1_000, ("zipf", 1.2)), (33, 1_000, "uniform")])
def test_crossprod_two_table_star_in_join_order(il, c_S, r_R, dist):
    # entity tables of up to 32 columns give S^T S and the per-row sums of S from one pass in join order:
    # one and two column tiles, unaligned rows (5, 17, 31), a ragged last tile of R, heavy keys spanning many
    # batches, rows of R nobody joins; 33 columns fall back to the block-by-block path
    rng = datagen.rng_for(1300 + c_S)
    sch = datagen.star_schema(rng, 7_003, c_S, [(r_R, 24, dist)])
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    G1 = il.ilargi_crossprod(plan).cpu().numpy()
    il.ilargi_plan_trace_begin(plan, "*", 64)
    G2 = il.ilargi_crossprod(plan).cpu().numpy()
    _, names = il.ilargi_plan_trace_end(plan, 64, names=True)
    assert rel(G1, oracle.crossprod(tg)) < OP_TOL
    assert np.array_equal(G1, G1.T) and np.array_equal(G1, G2)
    longest = np.bincount(sch.sources[1].row_idx, minlength=r_R).max()
    assert any(n.startswith("gram_star") for n in names) == (c_S <= 32 and longest <= 2048), (names, longest)


# ------------------------------------------------------------------ determinism and edge cases
def test_results_are_bitwise_reproducible(il):
    sch, tg, plan = get(il, "config2_small")
    rng = datagen.rng_for(8)
    Y = dev(rng.standard_normal((sch.r_T, 4)).astype(np.float32))
    X = dev(rng.standard_normal((sch.c_T, 4)).astype(np.float32))
    a1, b1, c1 = il.ilargi_tmm(plan, Y).cpu(), il.ilargi_lmm(plan, X).cpu(), il.ilargi_crossprod(plan).cpu()
    a2, b2, c2 = il.ilargi_tmm(plan, Y).cpu(), il.ilargi_lmm(plan, X).cpu(), il.ilargi_crossprod(plan).cpu()
    assert torch.equal(a1, a2) and torch.equal(b1, b2) and torch.equal(c1, c2)


def test_rows_without_any_source_and_unmapped_columns(il):
    rng = datagen.rng_for(13)
    r_T, c_T = 1_000, 9
    D = rng.standard_normal((50, 3)).astype(np.float32)
    idx = np.full(r_T, -1, dtype=np.int32)
    idx[100:200] = rng.integers(0, 50, 100)
    sch = datagen.Schema([datagen.Source(D, idx, np.array([7, -1, 2], dtype=np.int32))], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=2)
    T = il.ilargi_materialize(plan).cpu().numpy()
    assert np.array_equal(T, tg.T32) and np.all(T[:100] == 0) and np.all(T[:, [0, 1, 3, 4, 5, 6, 8]] == 0)
    X = rng.standard_normal((c_T, 2)).astype(np.float32)
    Y = rng.standard_normal((r_T, 2)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    got = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
    assert rel(got, oracle.tmm(tg, Y)) < OP_TOL and np.all(got[[0, 1, 3, 4, 5, 6, 8]] == 0)
    assert rel(il.ilargi_crossprod(plan).cpu().numpy(), oracle.crossprod(tg)) < OP_TOL


@pytest.mark.parametrize("r_T", [1, 63, 10_007])
def test_materialize_flat_stream_form(il, r_T):
    # aligned groups of four columns take the form that writes the table as one stream of float4: groups nobody
    # feeds (columns 0..3 and 28..31), an identity source shorter than the table, unmatched rows, a source column
    # offset inside the group tables (second source maps its columns 4..11 only), cells holding -0.0, ragged tail
    rng = datagen.rng_for(15 + r_T)
    c_T = 32
    n_a = max(1, (2 * r_T) // 3)
    A = rng.standard_normal((n_a, 8)).astype(np.float32)
    B = rng.standard_normal((37, 12)).astype(np.float32)
    A[rng.random(A.shape) < 0.1] = -0.0
    B[rng.random(B.shape) < 0.1] = -0.0
    idx_a = np.full(r_T, -1, dtype=np.int32)
    idx_a[:n_a] = np.arange(n_a)
    idx_b = rng.integers(0, 37, r_T).astype(np.int32)
    idx_b[rng.random(r_T) < 0.2] = -1
    map_b = np.array([-1, -1, -1, -1] + list(range(16, 24)), dtype=np.int32)
    sch = datagen.Schema([
        datagen.Source(A, idx_a, np.arange(4, 12, dtype=np.int32)),
        datagen.Source(B, idx_b, map_b),
    ], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=1)
    il.ilargi_plan_trace_begin(plan, "*", 8)
    T = il.ilargi_materialize(plan).cpu().numpy()
    il.ilargi_plan_trace_end(plan, 8)
    assert np.array_equal(T.view(np.uint32), tg.T32.view(np.uint32))
    assert not np.any(np.signbit(T[T == 0]))


def test_all_rows_unmatched_and_empty_sources(il):
    rng = datagen.rng_for(14)
    r_T, c_T = 300, 5
    S = rng.standard_normal((r_T, 2)).astype(np.float32)
    R = rng.standard_normal((10, 3)).astype(np.float32)
    none = np.full(r_T, -1, dtype=np.int32)
    empty_rows = np.zeros((0, 3), dtype=np.float32)
    sch = datagen.Schema([
        datagen.Source(S, None, np.array([0, 1], dtype=np.int32)),
        datagen.Source(R, none, np.array([2, 3, 4], dtype=np.int32)),
        datagen.Source(empty_rows, none.copy(), np.array([2, 3, 4], dtype=np.int32)),
    ], r_T, c_T)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=1)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy(), tg.T32)
    X = rng.standard_normal((c_T, 1)).astype(np.float32)
    Y = rng.standard_normal((r_T, 1)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_crossprod(plan).cpu().numpy(), oracle.crossprod(tg)) < OP_TOL


def test_index_out_of_range_is_reported(il):
    D = torch.zeros((10, 2), device="cuda")
    for bad in (10, -2):
        idx = np.zeros(100, dtype=np.int32)
        idx[57] = bad
        with pytest.raises(il.IlargiError) as ei:
            il.ilargi_plan_create([(D, dev(idx), np.array([0, 1], dtype=np.int32))], 100, 2, max_cx=1)
        assert ei.value.status == il.ERR_INDEX_RANGE


def test_operand_wider_than_plan_is_rejected(il):
    sch, tg, plan = get(il, "config0")
    X = torch.zeros((sch.c_T, 18), device="cuda")
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_lmm(plan, X)
    assert ei.value.status == il.ERR_WORKSPACE


def test_unaligned_table_pointer_falls_back_to_scalar_loads(il):
    # a table whose first element is only 4-byte aligned (a view one float into a buffer)
    rng = datagen.rng_for(15)
    r_T, r_k, c = 4_000, 300, 8
    S = rng.standard_normal((r_T, c)).astype(np.float32)
    R = rng.standard_normal((r_k, c)).astype(np.float32)
    fk = rng.integers(0, r_k, r_T).astype(np.int32)
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(c, 2 * c, dtype=np.int32))], r_T, 2 * c)
    tg = oracle.Target(sch)
    bufS = torch.empty(r_T * c + 1, device="cuda")
    bufR = torch.empty(r_k * c + 1, device="cuda")
    Sd = bufS[1:].view(r_T, c); Sd.copy_(dev(S))
    Rd = bufR[1:].view(r_k, c); Rd.copy_(dev(R))
    assert Sd.data_ptr() % 16 == 4
    plan = il.ilargi_plan_create([(Sd, None, sch.sources[0].col_map), (Rd, dev(fk), sch.sources[1].col_map)],
                                 r_T, 2 * c, max_cx=2)
    X = rng.standard_normal((2 * c, 2)).astype(np.float32)
    Y = rng.standard_normal((r_T, 2)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy(), tg.T32)


def test_sixteen_sources_with_shared_columns(il):
    # the largest source count the boundary accepts; columns shared by up to all of them, missing rows
    sch = datagen.tiny_random_schema(seed=77, r_T=2_503, c_T=23, n=16)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=16)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy(), tg.T32)
    rng = datagen.rng_for(78)
    for cx in (1, 16):
        X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_plan_create(il.schema_to_device(sch) + il.schema_to_device(sch)[:1], sch.r_T, sch.c_T, max_cx=1)
    assert ei.value.status == il.ERR_SHAPE


def test_source_with_the_maximum_column_count(il):
    # 4096 columns per source is the limit (one row of the operand slice must fit the LDS staging buffer)
    rng = datagen.rng_for(79)
    r_T, r_k, c = 257, 37, 4096
    R = rng.standard_normal((r_k, c)).astype(np.float32)
    S = rng.standard_normal((r_T, 3)).astype(np.float32)
    fk = rng.integers(0, r_k, r_T).astype(np.int32)
    sch = datagen.Schema([datagen.Source(S, None, np.arange(3, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(3, 3 + c, dtype=np.int32))], r_T, 3 + c)
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=16)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy(), tg.T32)
    for cx in (1, 3, 16):
        X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    too_wide = torch.zeros((r_k, c + 1), device="cuda")
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_plan_create([(too_wide, dev(fk), np.arange(c + 1, dtype=np.int32))], r_T, c + 1, max_cx=1)
    assert ei.value.status == il.ERR_UNSUPPORTED


def test_target_table_without_rows(il):
    # r_T = 0 (its buffers are empty, their pointers NULL): operators succeed and return empty or all-zero
    # results, the gradient step is refused
    D = torch.zeros((0, 2), device="cuda")
    plan = il.ilargi_plan_create([(D, None, np.array([0, 1], dtype=np.int32))], 0, 2, max_cx=2)
    assert il.ilargi_materialize(plan).shape == (0, 2)
    assert il.ilargi_lmm(plan, torch.ones((2, 2), device="cuda")).shape == (0, 2)
    out = torch.full((2, 2), 7.0, device="cuda")
    il.ilargi_tmm(plan, torch.zeros((0, 2), device="cuda"), out)
    assert torch.count_nonzero(out).item() == 0
    assert torch.count_nonzero(il.ilargi_crossprod(plan)).item() == 0
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_gd_step(plan, il.LINEAR, torch.zeros((2, 1), device="cuda"), torch.zeros(0, device="cuda"),
                          torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda"))
    assert ei.value.status == il.ERR_SHAPE


# ------------------------------------------------------------------ scalar operators (Tab. 2)
@pytest.mark.parametrize("name", ALL)
def test_row_sum_and_col_sum(il, name):
    sch, tg, plan = get(il, name)
    assert rel(il.ilargi_row_sum(plan).cpu().numpy(), oracle.row_sum(tg)) < OP_TOL
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(tg)) < OP_TOL


def _dense_after(il, sch, srcs, outs):
    """The table the result of an element-wise operator describes: same index arrays, new source tables."""
    plan2 = il.ilargi_plan_create([(o, idx, cm) for o, (_, idx, cm) in zip(outs, srcs)], sch.r_T, sch.c_T, max_cx=1)
    return il.ilargi_materialize(plan2).cpu().numpy()


ELEMENTWISE_CASES = [("mul", -1.75), ("div", 3.0), ("add", 0.5), ("sub", 2.0), ("pow", 3.0), ("pow", 0.5),
                     ("exp", 0.0), ("log", 0.0), ("sqrt", 0.0), ("abs", 0.0), ("square", 0.0)]


@pytest.mark.parametrize("op,x", ELEMENTWISE_CASES)
@pytest.mark.parametrize("maker", ["star", "star_unaligned"])
def test_elementwise_on_a_star_join(il, maker, op, x):
    # every target cell has exactly one source cell: all operators may act on the source tables
    rng = datagen.rng_for(1200)
    if maker == "star":
        sch = datagen.star_schema(rng, 20_011, 20, [(1_003, 200, "uniform"), (57, 8, ("zipf", 1.1))])
    else:
        sch = datagen.star_schema(rng, 3_001, 3, [(101, 7, "uniform")])
    if op in ("log", "sqrt") or (op == "pow" and x != int(x)):
        for s_ in sch.sources:
            s_.D[...] = np.abs(s_.D) + 0.25
    tg = oracle.Target(sch)
    srcs = il.schema_to_device(sch)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
    outs = il.ilargi_elementwise(plan, op, x)
    for o, (D, _, _) in zip(outs, srcs):
        assert o.data_ptr() != D.data_ptr()
    want = oracle.elementwise(tg, op, x)
    scale = float(np.abs(tg.T32).max()) + abs(x)
    np.testing.assert_allclose(_dense_after(il, sch, srcs, outs), want, rtol=2e-6, atol=2e-6 * scale)
    # in place: the same plan now describes the result
    il.ilargi_elementwise(plan, op, x, outs=[D for D, _, _ in srcs])
    np.testing.assert_allclose(il.ilargi_materialize(plan).cpu().numpy(), want, rtol=2e-6, atol=2e-6 * scale)
    assert rel(il.ilargi_row_sum(plan).cpu().numpy(), want.sum(axis=1)) < OP_TOL


def test_elementwise_conditions_on_shared_and_empty_cells(il):
    # shared columns and unmatched rows: only times and divide act on the sources alone
    sch, tg, plan = get(il, "tiny_mixed")
    srcs = il.schema_to_device(sch)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
    C = oracle.cover_counts(sch)
    assert C.max() > 1 and C.min() == 0
    for op, x in (("mul", 2.5), ("div", -4.0)):
        got = _dense_after(il, sch, srcs, il.ilargi_elementwise(plan, op, x))
        assert rel(got, oracle.elementwise(tg, op, x)) < 1e-6
    for op in ("add", "exp", "square", "abs"):
        with pytest.raises(il.IlargiError) as ei:
            il.ilargi_elementwise(plan, op, 1.0)
        assert ei.value.status == il.ERR_UNSUPPORTED
    # disjoint columns but rows without a match: operators that keep zero at zero are fine, the others not
    rng = datagen.rng_for(1201)
    sch2 = datagen.star_schema(rng, 2_003, 4, [(50, 6, "uniform")])
    sch2.sources[1].row_idx[::7] = -1
    tg2 = oracle.Target(sch2)
    srcs2 = il.schema_to_device(sch2)
    plan2 = il.ilargi_plan_create(srcs2, sch2.r_T, sch2.c_T, max_cx=1)
    assert oracle.cover_counts(sch2).max() == 1 and oracle.cover_counts(sch2).min() == 0
    for op, x in (("square", 0.0), ("abs", 0.0), ("pow", 2.0), ("mul", 3.0)):
        got = _dense_after(il, sch2, srcs2, il.ilargi_elementwise(plan2, op, x))
        np.testing.assert_allclose(got, oracle.elementwise(tg2, op, x), rtol=2e-6, atol=1e-6)
    for op, x in (("add", 1.0), ("exp", 0.0), ("log", 0.0), ("pow", -1.0), ("pow", 0.0)):
        with pytest.raises(il.IlargiError) as ei:
            il.ilargi_elementwise(plan2, op, x)
        assert ei.value.status == il.ERR_UNSUPPORTED
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_elementwise(plan2, 10, 0.0)
    assert ei.value.status == il.ERR_UNSUPPORTED


# ------------------------------------------------------------------ source tables in compressed sparse rows
def _sparse_case(il, name, p, which=True, max_cx=17):
    sch = datagen.sparsify(SCHEMAS[name](), p, seed=1300)
    tg = oracle.Target(sch)
    srcs = il.schema_to_device(sch, sparse=which)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=max_cx)
    return sch, tg, srcs, plan


@pytest.mark.parametrize("p", [0.0, 0.5, 0.9])
@pytest.mark.parametrize("name", ["config0", "config1_small", "config2_small", "config3_small", "tiny_mixed", "odd_cols"])
def test_sparse_sources_operators_and_join(il, name, p):
    # every table in compressed sparse rows (p = 0: all cells stored): join bit-exact, operators within the
    # float32 bound, row and column sums
    sch, tg, srcs, plan = _sparse_case(il, name, p)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy().view(np.uint32), tg.T32.view(np.uint32))
    rng = datagen.rng_for(1301)
    for cx in (1, 3, 4, 5, 17):
        X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_row_sum(plan).cpu().numpy(), oracle.row_sum(tg)) < OP_TOL
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(tg)) < OP_TOL
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)


@pytest.mark.parametrize("max_cx", [1, 3, 16, 40])
@pytest.mark.parametrize("which", [(0,), (1,)])
def test_sparse_sources_crossprod_mixed_tables_and_block_widths(il, which, max_cx):
    # one table sparse, one dense; the identity goes through in blocks of min(max_cx, 16) columns, with a ragged last block
    sch, tg, srcs, plan = _sparse_case(il, "config1_small", 0.8, which, max_cx=max_cx)
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    G2 = il.ilargi_crossprod(plan).cpu().numpy()
    assert np.array_equal(G, G2)


@pytest.mark.parametrize("which", [(0,), (1,), True])
@pytest.mark.parametrize("model", ["linear", "logistic"])
def test_sparse_sources_gradient_descent(il, model, which):
    # dense and sparse tables mixed: the entity table sparse (no shared pass), the dimension table sparse, both
    sch, tg, srcs, plan = _sparse_case(il, "config1_small", 0.7, which)
    rng = datagen.rng_for(1303)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(sch.r_T))
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    lrs = [0.05, 0.1, 0.2, 0.3, 0.4]
    W, L = _run_gd(il, plan, code, y, lrs, 10, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, len(lrs))), lrs, 10)
    assert max(rel(W[:, j], W_ref[:, j]) for j in range(len(lrs))) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


def test_sparse_sources_edge_cases(il):
    # empty rows and columns, a table without any stored entry, a long column split into chunks, unmatched rows
    rng = datagen.rng_for(1302)
    r_T = 9_001
    S = rng.standard_normal((r_T, 6)).astype(np.float32)
    S[:, 2] = 0.0                                    # an empty column
    S[100:300] = 0.0                                 # empty rows
    S[rng.random(S.shape) < 0.3] = 0.0
    R = np.zeros((40, 5), dtype=np.float32)          # no stored entry at all
    Q = rng.standard_normal((7, 3)).astype(np.float32)
    fk = rng.integers(0, 40, r_T).astype(np.int32)
    fq = rng.integers(0, 7, r_T).astype(np.int32)
    fq[::11] = -1
    sch = datagen.Schema([datagen.Source(S, None, np.arange(6, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(6, 11, dtype=np.int32)),
                          datagen.Source(Q, fq, np.array([11, -1, 12], dtype=np.int32))], r_T, 13)
    tg = oracle.Target(sch)
    srcs = il.schema_to_device(sch, sparse=True)
    assert srcs[1][0].nnz == 0 and srcs[0][0].nnz > 2 * 4096     # column chunks of 4096 entries
    plan = il.ilargi_plan_create(srcs, r_T, 13, max_cx=4)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy().view(np.uint32), tg.T32.view(np.uint32))
    X = rng.standard_normal((13, 4)).astype(np.float32)
    Y = rng.standard_normal((r_T, 4)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(tg)) < OP_TOL
    # element-wise operators act on the stored values; only those that keep zero at zero are accepted
    outs = il.ilargi_elementwise(plan, "square")
    for o, (D, _, _) in zip(outs, srcs):
        assert torch.equal(o, D.val * D.val)
    il.ilargi_elementwise(plan, "mul", -2.0, outs=[D.val for D, _, _ in srcs])      # in place
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), -2.0 * oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), -2.0 * oracle.lmm(tg, X)) < OP_TOL
    for op in ("exp", "add", "log"):
        with pytest.raises(il.IlargiError) as ei:
            il.ilargi_elementwise(plan, op, 1.0)
        assert ei.value.status == il.ERR_UNSUPPORTED
    G = il.ilargi_crossprod(plan).cpu().numpy()             # (values were scaled by -2 in place above)
    assert rel(G, 4.0 * oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    assert np.count_nonzero(G[2]) == 0 and np.count_nonzero(G[6:11]) == 0      # the empty column, the empty table
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_lmm(plan, torch.zeros((13, 4), device="cuda"), precision=il.BF16_IN_F32_ACC)
    assert ei.value.status == il.ERR_UNSUPPORTED


def test_sparse_table_wider_than_the_dense_limit(il):
    # a one-hot style dimension table with 10,000 columns and a few stored entries per row (dense tables stop at
    # 4096 columns): the operand is fetched per stored entry instead of being staged whole
    rng = datagen.rng_for(1303)
    r_T, r_R, c_S, c_R = 4_003, 1_501, 8, 10_000
    S = rng.standard_normal((r_T, c_S)).astype(np.float32)
    R = np.zeros((r_R, c_R), dtype=np.float32)
    for j in range(r_R):
        cols = rng.choice(c_R, size=int(rng.integers(0, 6)), replace=False)
        R[j, cols] = rng.standard_normal(cols.size).astype(np.float32)
    R[5, :1500] = 1.0                                   # one long row, still within the limit of such tables
    fk = rng.integers(0, r_R, r_T).astype(np.int32)
    fk[::13] = -1
    c_T = c_S + c_R
    sch = datagen.Schema([datagen.Source(S, None, np.arange(c_S, dtype=np.int32)),
                          datagen.Source(R, fk, np.arange(c_S, c_T, dtype=np.int32))], r_T, c_T)
    tg = oracle.Target(sch)
    srcs = il.schema_to_device(sch, sparse=[1])
    plan = il.ilargi_plan_create(srcs, r_T, c_T, max_cx=4)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy().view(np.uint32), tg.T32.view(np.uint32))
    for cx in (1, 3, 4):
        X = rng.standard_normal((c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_row_sum(plan).cpu().numpy(), oracle.row_sum(tg)) < OP_TOL
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(tg)) < OP_TOL
    w_star = rng.standard_normal(c_T)
    y = datagen.finish_labels("linear", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(r_T))
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.05], 5, c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((c_T, 1)), [0.05], 5)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)
    G = il.ilargi_crossprod(plan).cpu().numpy()             # 10,008 x 10,008, 2502 blocks of four identity columns
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    # the same table stored densely is refused, and so is a row with more entries than a staged block holds
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_plan_create(il.schema_to_device(sch), r_T, c_T, max_cx=1)
    assert ei.value.status == il.ERR_UNSUPPORTED
    R[7, :2100] = 1.0
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_plan_create(il.schema_to_device(sch, sparse=[1]), r_T, c_T, max_cx=1)
    assert ei.value.status == il.ERR_UNSUPPORTED


def test_one_hot_star_without_entity_table(il):
    # two joined one-hot style tables side by side and nothing else (the shape of the paper's real data sets,
    # Tab. 4, scaled down): no identity source to fuse, both tables in sparse rows
    tables, r_T, c_T = datagen.one_hot_star(9, 20_011, ((604, 951), (371, 384)), 20)
    sch = datagen.Schema([datagen.Source(t.dense(), t.row_idx, t.col_map) for t in tables], r_T, c_T)
    tg = oracle.Target(sch)
    srcs = [(il.CSR(dev(t.rowptr), dev(t.col), dev(t.val), (t.rows, t.cols)), dev(t.row_idx), t.col_map) for t in tables]
    plan = il.ilargi_plan_create(srcs, r_T, c_T, max_cx=4)
    assert np.array_equal(il.ilargi_materialize(plan).cpu().numpy().view(np.uint32), tg.T32.view(np.uint32))
    rng = datagen.rng_for(1304)
    for cx in (1, 4):
        X = rng.standard_normal((c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)
    w_star = rng.standard_normal(c_T)
    y = datagen.finish_labels("linear", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.01 * rng.standard_normal(r_T))
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.02], 6, c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((c_T, 1)), [0.02], 6)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=2e-4)


def test_sparse_crossprod_refuses_a_result_beyond_its_column_limit(il):
    # 20,000 target columns would need a 1.6 GB Gram matrix through 5000 rounds of multiplies: refused, nothing written
    r_T, c_T = 50, 20_000
    R = np.zeros((r_T, c_T), dtype=np.float32)
    R[np.arange(r_T), np.arange(r_T) * 7] = 1.0
    srcs = [(il.CSR.from_dense(R), None, np.arange(c_T, dtype=np.int32))]
    plan = il.ilargi_plan_create(srcs, r_T, c_T, max_cx=1)
    out = torch.zeros((4,), device="cuda")              # never touched: the call fails before any launch
    with pytest.raises(il.IlargiError) as ei:
        # (the binding would allocate c_T x c_T first: call the entry point itself)
        il._check(il.lib.ilargi_crossprod(plan.handle, out.data_ptr(), None), "ilargi_crossprod")
    assert ei.value.status == il.ERR_UNSUPPORTED
    assert torch.count_nonzero(out).item() == 0


def test_invalid_sparse_rows_are_reported(il):
    good = il.CSR.from_dense(np.array([[1.0, 0.0, 2.0], [0.0, 3.0, 0.0]], dtype=np.float32))
    cm = np.arange(3, dtype=np.int32)
    il.ilargi_plan_create([(good, None, cm)], 2, 3, max_cx=1)
    def broken(rowptr=None, col=None):
        return il.CSR(good.rowptr if rowptr is None else dev(np.array(rowptr, dtype=np.int32)),
                      good.col if col is None else dev(np.array(col, dtype=np.int32)), good.val, (2, 3))
    for bad in (broken(rowptr=[0, 3, 2]), broken(rowptr=[1, 2, 3]), broken(rowptr=[0, 2, 4]), broken(col=[0, 3, 1]),
                broken(col=[2, 0, 1]), broken(col=[0, 0, 1]), broken(col=[-1, 2, 1])):
        with pytest.raises(il.IlargiError) as ei:
            il.ilargi_plan_create([(bad, None, cm)], 2, 3, max_cx=1)
        assert ei.value.status == il.ERR_INDEX_RANGE


# ------------------------------------------------------------------ right multiply (Tab. 2, row XT)
@pytest.mark.parametrize("name", ["config0", "config1_small", "config3_small", "tiny_mixed", "odd_cols"])
@pytest.mark.parametrize("cx", [1, 2, 5, 16, 17])
def test_rmm(il, name, cx):
    sch, tg, plan = get(il, name)
    X = datagen.rng_for(1400 + cx).standard_normal((cx, sch.r_T)).astype(np.float32)
    assert rel(il.ilargi_rmm(plan, dev(X)).cpu().numpy(), oracle.rmm(tg, X)) < OP_TOL


def test_rmm_sparse_sources_and_wide_operand(il):
    sch, tg, srcs, plan = _sparse_case(il, "config1_small", 0.8)
    X = datagen.rng_for(1401).standard_normal((9, sch.r_T)).astype(np.float32)
    assert rel(il.ilargi_rmm(plan, dev(X)).cpu().numpy(), oracle.rmm(tg, X)) < OP_TOL
    sch, tg, plan = get(il, "config1_small", max_cx=256)
    X = datagen.rng_for(1402).standard_normal((100, sch.r_T)).astype(np.float32)
    assert rel(il.ilargi_rmm(plan, dev(X)).cpu().numpy(), oracle.rmm(tg, X)) < OP_TOL
    e = rel(il.ilargi_rmm(plan, dev(X), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.rmm(tg, X))
    assert e < BF16_TOL


# ------------------------------------------------------------------ calibration kernels
@pytest.mark.parametrize("blocks", [1, 8192, None])
def test_stream_probe_copies_reads_and_writes_whole_buffers(il, blocks):
    # the plain streaming kernels behind the bench's bandwidth figures and the counter scaling: a copy moves every
    # float, the write fills every float, whatever the launch shape (None: one float4 per thread, in address order)
    n = 4 * 1_000_003                                    # not a multiple of the workgroup size
    nb = n // 1024 + 1 if blocks is None else blocks
    src = torch.arange(n, device="cuda", dtype=torch.float32)
    dst = torch.zeros(n, device="cuda")
    for kind in (0, 3):
        dst.zero_()
        il.ilargi_stream_probe(kind, dst, src, n, nb)
        assert torch.equal(dst, src)
    for kind in (2, 4):
        dst.zero_()
        il.ilargi_stream_probe(kind, dst, None, n, nb)
        assert torch.equal(dst.view(-1, 4), torch.tensor([1.0, 2.0, 3.0, 4.0], device="cuda").expand(n // 4, 4))
    sink = torch.zeros(nb, device="cuda")
    il.ilargi_stream_probe(1, sink, torch.ones(n, device="cuda"), n, nb)
    assert sink.sum().item() > 0.0
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_stream_probe(0, dst, src, n, (1 << 22) + 1)
    assert ei.value.status == il.ERR_SHAPE


# ------------------------------------------------------------------ streams
def test_calls_on_a_side_stream(il):
    # everything a call enqueues goes to the stream it is given: results are right when the caller only
    # synchronizes that stream, with unrelated work on the default stream in between
    sch = datagen.config1(r_S=50_021, r_R=5_003, c_R=200)
    tg = oracle.Target(sch)
    side = torch.cuda.Stream()
    rng = datagen.rng_for(1500)
    X = dev(rng.standard_normal((sch.c_T, 3)).astype(np.float32))
    Y = dev(rng.standard_normal((sch.r_T, 3)).astype(np.float32))
    X64 = dev(rng.standard_normal((sch.c_T, 64)).astype(np.float32))
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=64)
        noise = torch.randn(4096, 4096, device="cuda")
        a = il.ilargi_lmm(plan, X)
        b = il.ilargi_tmm(plan, Y)
        c = il.ilargi_lmm(plan, X64)
        g = il.ilargi_crossprod(plan)
        t = il.ilargi_materialize(plan)
    torch.cuda.default_stream().wait_stream(side)       # the default stream only orders itself after the side stream
    _ = (noise @ noise).sum()
    side.synchronize()
    assert rel(a.cpu().numpy(), oracle.lmm(tg, X.cpu().numpy())) < OP_TOL
    assert rel(b.cpu().numpy(), oracle.tmm(tg, Y.cpu().numpy())) < OP_TOL
    assert rel(c.cpu().numpy(), oracle.lmm(tg, X64.cpu().numpy())) < OP_TOL
    assert rel(g.cpu().numpy(), oracle.crossprod(tg)) < OP_TOL
    assert np.array_equal(t.cpu().numpy(), tg.T32)
