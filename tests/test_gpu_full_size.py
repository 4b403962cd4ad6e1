"""The five benchmark configurations at their full sizes, device library against the CPU oracle.

Operators are compared with the oracle computed on the spot (one materialization per configuration,
shared by the tests of that configuration).  The long gradient-descent runs are compared with
expectations the oracle wrote beforehand (tests/golden/*.npz, produced by tests/golden/make_golden.py,
which calls only the generators and the oracle); a checksum of the labels proves that the device is
given the same problem.
"""
import hashlib
import os

import numpy as np
import pytest

import datagen
import oracle
from tolerances import bf16_gd_weight_tol, lambda_max

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

torch = pytest.importorskip("torch")

OP_TOL = 1e-5
GD_TOL = 1e-4
BF16_OP_TOL = 5e-3
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def il():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_01985_amd as mod
    return mod


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


class Problem:
    """Schema, oracle table, device plan and labels of one configuration (built once per module)."""
    cache = {}

    @classmethod
    def get(cls, il, name, max_cx, kind=None):
        if name not in cls.cache:
            cls.cache.clear()          # one configuration resident at a time (host and device memory)
            torch.cuda.empty_cache()
            sch = getattr(datagen, name)()
            tg = oracle.Target(sch)
            plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=max_cx)
            y = None
            if kind is not None:
                y = datagen.finish_labels(kind, oracle.lmm(tg, sch.extras["w_star"].reshape(-1, 1)), sch.extras["noise"])
            cls.cache[name] = (sch, tg, plan, y)
        return cls.cache[name]


def run_gd(il, plan, model, y, lrs, iters, c_T, precision=0):
    m = len(lrs)
    W = torch.zeros((c_T, m), device="cuda")
    lr = dev(np.asarray(lrs, dtype=np.float32))
    loss = torch.zeros(m, device="cuda")
    yd = dev(y)
    losses = []
    for _ in range(iters):
        il.ilargi_gd_step(plan, model, W, yd, lr, loss, precision=precision)
        losses.append(loss.cpu().numpy().copy())
    return W.cpu().numpy(), np.array(losses)


def check_ops(il, sch, tg, plan, widths):
    rng = datagen.rng_for(4242)
    for cx in widths:
        X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
        Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
        assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL, ("lmm", cx)
        assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL, ("tmm", cx)


# ------------------------------------------------------------------ configuration 1 (operator micro-benchmark)
def test_config1_operators_and_join(il):
    sch, tg, plan, _ = Problem.get(il, "config1", 16)
    T = il.ilargi_materialize(plan)
    assert torch.equal(T.cpu().view(torch.int32), torch.from_numpy(tg.T32).view(torch.int32))
    del T
    for key, fn, ofn in (("X1", il.ilargi_lmm, oracle.lmm), ("X16", il.ilargi_lmm, oracle.lmm),
                         ("Y1", il.ilargi_tmm, oracle.tmm), ("Y16", il.ilargi_tmm, oracle.tmm)):
        got = fn(plan, dev(sch.extras[key])).cpu().numpy()
        assert rel(got, ofn(tg, sch.extras[key])) < OP_TOL, key
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, oracle.crossprod(tg)) < OP_TOL and np.array_equal(G, G.T)


def test_config1_materialized_plan_agrees(il):
    # the baseline strategy: join once, then dense operators on T through the same entry points
    sch, tg, plan, _ = Problem.get(il, "config1", 16)
    T = il.ilargi_materialize(plan)
    mplan = il.ilargi_plan_create([(T, None, np.arange(sch.c_T, dtype=np.int32))], sch.r_T, sch.c_T, max_cx=16)
    X, Y = sch.extras["X16"], sch.extras["Y16"]
    assert rel(il.ilargi_lmm(mplan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(mplan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL
    assert rel(il.ilargi_tmm(mplan, dev(sch.extras["Y1"])).cpu().numpy(), oracle.tmm(tg, sch.extras["Y1"])) < OP_TOL


def test_config1_kmeans_and_gaussian_nmf(il):
    # the two unsupervised models at full size, ten centroids / rank ten, one step each from given values
    sch, tg, plan, _ = Problem.get(il, "config1", 16)
    rng = datagen.rng_for(77)
    C0 = np.ascontiguousarray(tg.T32[rng.choice(sch.r_T, 10, replace=False)].T)
    C = dev(C0)
    assign = torch.empty(sch.r_T, dtype=torch.int32, device="cuda")
    counts = torch.empty(10, dtype=torch.int32, device="cuda")
    il.ilargi_kmeans_step(plan, C, assign, counts)
    C_ref, a_ref, n_ref, _ = oracle.kmeans_step(tg, C0)
    a = assign.cpu().numpy()
    differ = np.flatnonzero(a != a_ref)
    assert differ.size <= 20, differ.size                       # near-ties in float32 only
    if differ.size:
        d2 = oracle.kmeans_distances(oracle.Target(table=tg.T32[differ]), C0)
        gap = d2[np.arange(differ.size), a[differ]] - d2[np.arange(differ.size), a_ref[differ]]
        assert np.all(gap <= 2e-6 * d2.max(axis=1))
    assert np.array_equal(counts.cpu().numpy(), np.bincount(a, minlength=10))
    assert rel(C.cpu().numpy(), C_ref) < (OP_TOL if differ.size == 0 else GD_TOL)
    # Gaussian NMF needs a non-negative table: the same schema with absolute values
    for s in sch.sources:
        s.D[...] = np.abs(s.D)
    tg2 = oracle.Target(sch)
    plan2 = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=10)
    W0 = (rng.random((sch.r_T, 10)) + 0.05).astype(np.float32)
    H0 = (rng.random((10, sch.c_T)) + 0.05).astype(np.float32)
    W, Ht = dev(W0), dev(np.ascontiguousarray(H0.T))
    il.ilargi_gnmf_step(plan2, W, Ht)
    W_ref, H_ref = oracle.gnmf_step(tg2, W0, H0)
    assert rel(W.cpu().numpy(), W_ref) < OP_TOL and rel(Ht.cpu().numpy().T, H_ref) < OP_TOL
    Problem.cache.clear()                                       # the cached schema was changed in place


def test_config1_gradient_descent_on_the_clustered_entity_table(il):
    # the benchmark's schema at full size: the one-pass iteration over the join-ordered copy (linear and logistic, five
    # iterations each) against the oracle's Alg. 1, and the Gram matrix bit for bit against the plan without the copy
    sch, tg, plan, _ = Problem.get(il, "config1", 16)
    rng = datagen.rng_for(4711)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    G0 = il.ilargi_crossprod(plan).cpu().numpy()
    for model, code, lr in (("linear", il.LINEAR, 0.05), ("logistic", il.LOGISTIC, 0.5)):
        y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(sch.r_T))
        yd = dev(y)
        il.ilargi_plan_cluster(plan, y=yd)
        W = torch.zeros((sch.c_T, 1), device="cuda")
        lrd = dev(np.array([lr], dtype=np.float32))
        loss = torch.zeros(1, device="cuda")
        losses = []
        for _ in range(5):
            il.ilargi_gd_step(plan, code, W, yd, lrd, loss)
            losses.append(loss.cpu().numpy().copy())
        W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 1)), [lr], 5)
        assert rel(W.cpu().numpy(), W_ref) < GD_TOL, model
        np.testing.assert_allclose(np.array(losses), L_ref, rtol=1e-4)
    G1 = il.ilargi_crossprod(plan).cpu().numpy()
    assert np.array_equal(G0, G1)
    il.ilargi_plan_cluster(plan, None)


# ------------------------------------------------------------------ configuration 2 (logistic regression, Zipf keys)
def test_config1_scalar_operators(il):
    # Tab. 2, first four rows, at full size: sums against the oracle; an element-wise operator applied to the
    # sources, checked on the table it describes (a sample of rows through the oracle, cell by cell)
    sch, tg, plan, _ = Problem.get(il, "config1", 16)
    assert rel(il.ilargi_row_sum(plan).cpu().numpy(), oracle.row_sum(tg)) < OP_TOL
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(tg)) < OP_TOL
    srcs = il.schema_to_device(sch)
    plan2 = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
    outs = il.ilargi_elementwise(plan2, "exp", 0.0)
    plan3 = il.ilargi_plan_create([(o, idx, cm) for o, (_, idx, cm) in zip(outs, srcs)], sch.r_T, sch.c_T, max_cx=1)
    T2 = il.ilargi_materialize(plan3)
    rows = datagen.rng_for(5).integers(0, sch.r_T, 4_000)
    want = oracle.apply_elementwise(tg.T32[rows], "exp")
    np.testing.assert_allclose(T2[torch.from_numpy(rows).cuda()].cpu().numpy(), want, rtol=2e-6)


def test_config2_logistic_regression(il):
    sch, tg, plan, y = Problem.get(il, "config2", 16, "logistic")
    gold = np.load(os.path.join(GOLDEN, "config2_gd.npz"))
    assert sha(y) == str(gold["y_sha256"])
    cnt = np.bincount(sch.sources[2].row_idx, minlength=sch.sources[2].rows)
    assert cnt.max() > 500_000          # the heavy key of the Zipf law: one very long inverse-index segment
    W, L = run_gd(il, plan, il.LOGISTIC, y, [0.5], 50, sch.c_T)
    assert rel(W, gold["W"]) < GD_TOL
    np.testing.assert_allclose(L, gold["losses"], rtol=1e-4)


def test_config2_operators(il):
    sch, tg, plan, _ = Problem.get(il, "config2", 16, "logistic")
    check_ops(il, sch, tg, plan, [1, 3, 16])
    rowptr, perm = il.ilargi_plan_inverse_index(plan, 2)
    idx = sch.sources[2].row_idx
    assert np.array_equal(np.diff(rowptr), np.bincount(idx, minlength=sch.sources[2].rows))
    assert np.array_equal(perm, np.argsort(idx, kind="stable").astype(np.int32))


# ------------------------------------------------------------------ configuration 3 (union with overlap)
def test_config3_gram_and_linear_regression(il):
    sch, tg, plan, y = Problem.get(il, "config3", 16, "linear")
    gold = np.load(os.path.join(GOLDEN, "config3_gd.npz"))
    assert sha(y) == str(gold["y_sha256"])
    G = il.ilargi_crossprod(plan).cpu().numpy()
    assert rel(G, gold["gram"]) < OP_TOL and np.array_equal(G, G.T)
    W, L = run_gd(il, plan, il.LINEAR, y, [0.1], 10, sch.c_T)
    assert rel(W, gold["W"]) < GD_TOL
    np.testing.assert_allclose(L, gold["losses"], rtol=1e-4)


def test_config3_operators_and_join(il):
    sch, tg, plan, _ = Problem.get(il, "config3", 16, "linear")
    check_ops(il, sch, tg, plan, [1, 4, 16])
    T = il.ilargi_materialize(plan)
    assert torch.equal(T.cpu().view(torch.int32), torch.from_numpy(tg.T32).view(torch.int32))


# ------------------------------------------------------------------ configuration 4 (256 models at once)
def test_config4_batched_models_fp32(il):
    sch, tg, plan, y = Problem.get(il, "config4", 256, "linear")
    gold = np.load(os.path.join(GOLDEN, "config4_gd.npz"))
    assert sha(y) == str(gold["y_sha256"])
    lrs = sch.extras["lr"]
    W, L = run_gd(il, plan, il.LINEAR, y, lrs, 20, sch.c_T)
    errs = np.array([rel(W[:, j], gold["W"][:, j]) for j in range(256)])
    assert errs.max() < GD_TOL, (errs.max(), int(errs.argmax()))
    np.testing.assert_allclose(L, gold["losses"], rtol=2e-4)


def test_config4_wide_operators_fp32(il):
    sch, tg, plan, _ = Problem.get(il, "config4", 256, "linear")
    rng = datagen.rng_for(99)
    X = rng.standard_normal((sch.c_T, 256)).astype(np.float32)
    Y = rng.standard_normal((sch.r_T, 256)).astype(np.float32)
    assert rel(il.ilargi_lmm(plan, dev(X)).cpu().numpy(), oracle.lmm(tg, X)) < OP_TOL
    assert rel(il.ilargi_tmm(plan, dev(Y)).cpu().numpy(), oracle.tmm(tg, Y)) < OP_TOL


def test_config4_bf16_inputs(il):
    sch, tg, plan, y = Problem.get(il, "config4", 256, "linear")
    gold = np.load(os.path.join(GOLDEN, "config4_gd.npz"))
    rng = datagen.rng_for(99)
    X = rng.standard_normal((sch.c_T, 256)).astype(np.float32)
    Y = rng.standard_normal((sch.r_T, 256)).astype(np.float32)
    e1 = rel(il.ilargi_lmm(plan, dev(X), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.lmm(tg, X))
    e2 = rel(il.ilargi_tmm(plan, dev(Y), precision=il.BF16_IN_F32_ACC).cpu().numpy(), oracle.tmm(tg, Y))
    assert e1 < BF16_OP_TOL and e2 < BF16_OP_TOL, (e1, e2)
    # weights under bfloat16 inputs: the bound derived in tests/tolerances.py, per model
    W, L = run_gd(il, plan, il.LINEAR, y, sch.extras["lr"], 20, sch.c_T, precision=il.BF16_IN_F32_ACC)
    errs = np.array([rel(W[:, j], gold["W"][:, j]) for j in range(256)])
    print(f"bf16-input GD, 256 models: max relative weight error {errs.max():.3e}, median {np.median(errs):.3e}")
    lam = lambda_max(oracle.crossprod(tg), sch.r_T)
    tols = np.array([bf16_gd_weight_tol(20, sch.c_T, sch.r_T, lr_j, lam) for lr_j in sch.extras["lr"]])
    print(f"  bound {tols.min():.3e} .. {tols.max():.3e} (lambda_max {lam:.4f})")
    assert np.all(errs < tols), (errs / tols).max()


def test_config4_batched_models_on_the_clustered_entity_table(il):
    # 256 models at full size with the fused pass streaming the join-ordered copy, its keys and labels: the same bits
    # as the pass that gathers the rows, in both precisions, and the oracle's weights in float32
    sch, tg, plan, y = Problem.get(il, "config4", 256, "linear")
    gold = np.load(os.path.join(GOLDEN, "config4_gd.npz"))
    lrs = sch.extras["lr"]
    yd, lr = dev(y), dev(np.asarray(lrs, dtype=np.float32))

    def run(precision):
        W = torch.zeros((sch.c_T, 256), device="cuda")
        loss = torch.zeros(256, device="cuda")
        for _ in range(20):
            il.ilargi_gd_step(plan, il.LINEAR, W, yd, lr, loss, precision=precision)
        return W.cpu().numpy(), loss.cpu().numpy()

    plain = {p: run(p) for p in (il.F32, il.BF16_IN_F32_ACC)}
    il.ilargi_plan_cluster(plan, y=yd)
    for p in (il.F32, il.BF16_IN_F32_ACC):
        W, L = run(p)
        assert np.array_equal(W, plain[p][0]) and np.array_equal(L, plain[p][1])
    errs = np.array([rel(plain[il.F32][0][:, j], gold["W"][:, j]) for j in range(256)])
    assert errs.max() < GD_TOL
    il.ilargi_plan_cluster(plan, None)


def test_sliced_segment_sums_on_a_large_target_table(il):
    # target tables from 1.5 million rows on split every segment of the inverse index by slice of target rows
    # (narrow transposed multiply and gradient descent); a Zipf key gives runs far beyond the long-segment limit in
    # every slice, the second table has rows with entries in only some slices, the third is a tiny one
    rng = datagen.rng_for(8100)
    sch = datagen.star_schema(rng, 1_600_037, 4, [(1_000, 8, ("zipf", 1.3)), (150_000, 4, "uniform"), (37, 5, "uniform")])
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=4)
    for cx in (1, 3, 4):
        Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
        got = il.ilargi_tmm(plan, dev(Y)).cpu().numpy()
        assert rel(got, oracle.tmm(tg, Y)) < OP_TOL
        assert np.array_equal(got, il.ilargi_tmm(plan, dev(Y)).cpu().numpy())          # same bits on every run
    assert rel(il.ilargi_col_sum(plan).cpu().numpy(), oracle.col_sum(sch)) < OP_TOL
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels("logistic", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(sch.r_T))
    W = torch.zeros((sch.c_T, 1), device="cuda")
    lr = dev(np.array([0.5], dtype=np.float32))
    loss = torch.zeros(1, device="cuda")
    losses = []
    for _ in range(5):
        il.ilargi_gd_step(plan, il.LOGISTIC, W, dev(y), lr, loss)
        losses.append(float(loss.item()))
    W_ref, L_ref = oracle.gd(tg, "logistic", y, np.zeros((sch.c_T, 1)), [0.5], 5)
    assert rel(W.cpu().numpy(), W_ref) < GD_TOL
    np.testing.assert_allclose(np.array(losses), L_ref[:, 0], rtol=1e-4)
