"""KMeans and Gaussian NMF steps of the device library against the CPU oracle.

Both are compositions of the left and the transposed multiply with row-local steps; the tolerances are the
ones of those operators (1e-5 relative Frobenius error for one step, 1e-4 for chains of steps).  The KMeans
assignment is an integer decided by float32 arithmetic on the device and by float64 in the oracle: rows may
differ only where the oracle's two distances agree to float32 accuracy, and the tests say how many did.
"""
import numpy as np
import pytest

import datagen
import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

OP_TOL = 1e-5
CHAIN_TOL = 1e-4


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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


SCHEMAS = {
    "config0": lambda: datagen.config0(),
    "config1_small": lambda: datagen.config1(r_S=30_011, r_R=3_001, c_R=200),
    "config2_small": lambda: datagen.config2(r_S=100_003, dim_rows=(4_000, 2_000, 400)),
    "config3_small": lambda: datagen.config3(rows=50_001, cols=64, shared=32),
    "tiny_mixed": lambda: datagen.tiny_random_schema(21, r_T=333, c_T=19, n=5),
    "odd_cols": lambda: datagen.star_schema(datagen.rng_for(77), 5_001, 7, [(97, 13, "uniform"), (31, 2, "uniform")]),
}
_cache = {}


def get(il, name, nonneg=False, sparse=False):
    key = (name, nonneg, sparse)
    if key not in _cache:
        sch = SCHEMAS[name]()
        if nonneg:
            for s in sch.sources:
                s.D[...] = np.abs(s.D)
        if sparse:
            sch = datagen.sparsify(sch, 0.7, seed=1400)
        tg = oracle.Target(sch)
        plan = il.ilargi_plan_create(il.schema_to_device(sch, sparse=sparse), sch.r_T, sch.c_T, max_cx=64)
        _cache[key] = (sch, tg, plan)
    return _cache[key]


# ------------------------------------------------------------------ KMeans
def start_centroids(tg, k, seed):
    rng = datagen.rng_for(seed)
    rows = rng.choice(tg.r_T, size=k, replace=tg.r_T < k)
    C = tg.T32[rows].astype(np.float64).T + 0.01 * rng.standard_normal((tg.c_T, k))
    return np.ascontiguousarray(C.astype(np.float32))


def check_kmeans_step(il, tg, plan, C0):
    """One device step from C0 against one oracle step from C0; returns the device's new centroids."""
    k = C0.shape[1]
    C = dev(C0)
    assign = torch.full((tg.r_T,), -1, dtype=torch.int32, device="cuda")
    counts = torch.full((k,), -1, dtype=torch.int32, device="cuda")
    il.ilargi_kmeans_step(plan, C, assign, counts)
    C_ref, a_ref, n_ref, _ = oracle.kmeans_step(tg, C0)
    a = assign.cpu().numpy()
    n = counts.cpu().numpy()
    assert a.min() >= 0 and a.max() < k
    assert np.array_equal(n, np.bincount(a, minlength=k))            # sizes are exact for the device's own assignment
    differ = np.flatnonzero(a != a_ref)
    if differ.size:
        # allowed only where float32 cannot tell the two centroids apart
        d2 = oracle.kmeans_distances(oracle.Target(table=tg.T32[differ]), C0)
        gap = d2[np.arange(differ.size), a[differ]] - d2[np.arange(differ.size), a_ref[differ]]
        scale = (tg.T32[differ].astype(np.float64) ** 2).sum(axis=1) + (C0.astype(np.float64) ** 2).sum(axis=0).max()
        assert np.all(gap <= 2e-6 * scale), (differ.size, float((gap / scale).max()))
        assert differ.size <= max(1, tg.r_T // 10_000), differ.size
    got = C.cpu().numpy()
    same = np.ones(k, dtype=bool)
    same[a[differ]] = False
    same[a_ref[differ]] = False
    assert same.sum() >= k - 2 * differ.size
    if same.any():
        assert rel(got[:, same], C_ref[:, same]) < OP_TOL
    empty = n_ref == 0
    assert np.array_equal(got[:, empty & same], C0[:, empty & same])  # untouched, bit for bit
    return got, differ.size


@pytest.mark.parametrize("k", [1, 3, 10, 17, 64])
@pytest.mark.parametrize("name", list(SCHEMAS))
def test_kmeans_step(il, name, k):
    sch, tg, plan = get(il, name)
    check_kmeans_step(il, tg, plan, start_centroids(tg, k, 100 + k))


@pytest.mark.parametrize("name", ["config1_small", "config2_small"])
def test_kmeans_iterations_follow_the_oracle(il, name):
    sch, tg, plan = get(il, name)
    C_dev = start_centroids(tg, 8, 7)
    C_ref = C_dev.astype(np.float64)
    mismatches = 0
    for _ in range(5):
        C_ref = oracle.kmeans_step(tg, C_ref)[0]
        C_dev, d = check_kmeans_step(il, tg, plan, C_dev)
        mismatches += d
    if mismatches == 0:
        assert rel(C_dev, C_ref) < CHAIN_TOL


def test_kmeans_empty_cluster_duplicate_centroid_and_optional_outputs(il):
    sch, tg, plan = get(il, "config1_small")
    C0 = start_centroids(tg, 5, 11)
    C0[:, 3] = C0[:, 1]                       # a duplicate: ties go to the first
    C0[:, 4] = 1e4                            # nobody is near
    C = dev(C0)
    counts = torch.zeros(5, dtype=torch.int32, device="cuda")
    il.ilargi_kmeans_step(plan, C, None, counts)
    n = counts.cpu().numpy()
    C_ref, a_ref, n_ref, _ = oracle.kmeans_step(tg, C0)
    assert n[3] == 0 and n[4] == 0 and n.sum() == tg.r_T and np.array_equal(n, n_ref)
    got = C.cpu().numpy()
    assert np.array_equal(got[:, 3:], C0[:, 3:])
    assert rel(got[:, :3], C_ref[:, :3]) < OP_TOL
    C2 = dev(C0)
    il.ilargi_kmeans_step(plan, C2)           # no optional outputs at all
    assert torch.equal(C, C2)


def test_kmeans_sparse_sources(il):
    sch, tg, plan = get(il, "config1_small", sparse=True)
    check_kmeans_step(il, tg, plan, start_centroids(tg, 6, 21))


def test_kmeans_limits_are_reported(il):
    sch, tg, plan = get(il, "tiny_mixed")
    with pytest.raises(RuntimeError, match="WORKSPACE"):
        il.ilargi_kmeans_step(plan, torch.zeros((tg.c_T, 65), device="cuda"))
    big = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=300)
    with pytest.raises(RuntimeError, match="UNSUPPORTED"):
        il.ilargi_kmeans_step(big, torch.zeros((tg.c_T, 257), device="cuda"))
    C0 = start_centroids(tg, 256, 5)
    check_kmeans_step(il, tg, big, C0)        # the largest supported number of centroids


# ------------------------------------------------------------------ Gaussian NMF
def start_factors(tg, r, seed):
    rng = datagen.rng_for(seed)
    W = (rng.random((tg.r_T, r)) + 0.05).astype(np.float32)
    H = (rng.random((r, tg.c_T)) + 0.05).astype(np.float32)
    return W, H


def device_gnmf(il, plan, W, H, steps=1):
    Wd, Htd = dev(W), dev(np.ascontiguousarray(H.T))
    for _ in range(steps):
        il.ilargi_gnmf_step(plan, Wd, Htd)
    return Wd.cpu().numpy(), Htd.cpu().numpy().T


@pytest.mark.parametrize("r", [1, 3, 10, 17, 64])
@pytest.mark.parametrize("name", list(SCHEMAS))
def test_gnmf_step(il, name, r):
    sch, tg, plan = get(il, name, nonneg=True)
    W, H = start_factors(tg, r, 200 + r)
    W1, H1 = device_gnmf(il, plan, W, H)
    W_ref, H_ref = oracle.gnmf_step(tg, W, H)
    assert rel(W1, W_ref) < OP_TOL and rel(H1, H_ref) < OP_TOL
    assert W1.min() >= 0.0 and H1.min() >= 0.0


@pytest.mark.parametrize("name", ["config1_small", "config3_small"])
def test_gnmf_iterations_follow_the_oracle_and_lower_the_objective(il, name):
    sch, tg, plan = get(il, name, nonneg=True)
    W, H = start_factors(tg, 5, 31)
    W_ref, H_ref = W.astype(np.float64), H.astype(np.float64)
    first = oracle.gnmf_objective(tg, W, H)
    for _ in range(10):
        W_ref, H_ref = oracle.gnmf_step(tg, W_ref, H_ref)
    W1, H1 = device_gnmf(il, plan, W, H, steps=10)
    assert rel(W1, W_ref) < CHAIN_TOL and rel(H1, H_ref) < CHAIN_TOL
    assert oracle.gnmf_objective(tg, W1, H1) < first
    np.testing.assert_allclose(oracle.gnmf_objective(tg, W1, H1), oracle.gnmf_objective(tg, W_ref, H_ref), rtol=1e-4)


def test_gnmf_zero_rows_and_columns_and_exact_factorization(il):
    sch, tg, plan = get(il, "config0", nonneg=True)
    W, H = start_factors(tg, 4, 41)
    W[7] = 0.0
    H[:, 3] = 0.0
    W1, H1 = device_gnmf(il, plan, W, H)
    W_ref, H_ref = oracle.gnmf_step(tg, W, H)
    assert np.all(np.isfinite(W1)) and np.all(np.isfinite(H1))
    assert np.all(W1[7] == 0.0) and np.all(H1[:, 3] == 0.0)
    assert rel(W1, W_ref) < OP_TOL and rel(H1, H_ref) < OP_TOL
    # a table that is exactly W H (small integers) is a fixed point
    rng = datagen.rng_for(42)
    Wi = rng.integers(1, 5, (1_000, 3)).astype(np.float32)
    Hi = rng.integers(1, 5, (3, 8)).astype(np.float32)
    table = Wi @ Hi
    p2 = il.ilargi_plan_create([(dev(table), None, np.arange(8, dtype=np.int32))], 1_000, 8, max_cx=4)
    W2, H2 = device_gnmf(il, p2, Wi, Hi)
    np.testing.assert_allclose(W2, Wi, rtol=2e-6)
    np.testing.assert_allclose(H2, Hi, rtol=2e-6)


def test_gnmf_sparse_sources_and_limits(il):
    sch, tg, plan = get(il, "config1_small", nonneg=True, sparse=True)
    W, H = start_factors(tg, 6, 51)
    W1, H1 = device_gnmf(il, plan, W, H)
    W_ref, H_ref = oracle.gnmf_step(tg, W, H)
    assert rel(W1, W_ref) < OP_TOL and rel(H1, H_ref) < OP_TOL
    small = get(il, "tiny_mixed")[0]
    big = il.ilargi_plan_create(il.schema_to_device(small), small.r_T, small.c_T, max_cx=128)
    with pytest.raises(RuntimeError, match="UNSUPPORTED"):
        il.ilargi_gnmf_step(big, torch.ones((small.r_T, 65), device="cuda"), torch.ones((small.c_T, 65), device="cuda"))
    with pytest.raises(RuntimeError, match="WORKSPACE"):
        il.ilargi_gnmf_step(plan, torch.ones((tg.r_T, 65), device="cuda"), torch.ones((tg.c_T, 65), device="cuda"))


def test_models_on_a_target_table_without_rows(il):
    # r_T = 0: KMeans leaves the centroids where they are and reports empty clusters; the NMF round multiplies
    # H by 0 / tiny (the numerator T^T W is zero), and W has no rows to update
    D = torch.zeros((0, 3), device="cuda")
    plan = il.ilargi_plan_create([(D, None, np.arange(3, dtype=np.int32))], 0, 3, max_cx=2)
    C0 = torch.tensor([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]], device="cuda")
    C = C0.clone()
    counts = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    assign = torch.zeros(0, dtype=torch.int32, device="cuda")
    il.ilargi_kmeans_step(plan, C, assign, counts)
    assert torch.equal(C, C0) and counts.cpu().tolist() == [0, 0]
    W = torch.zeros((0, 2), device="cuda")
    Ht = torch.ones((3, 2), device="cuda")
    il.ilargi_gnmf_step(plan, W, Ht)
    assert torch.count_nonzero(Ht).item() == 0           # H o (W^T T) / max(W^T W H, tiny) with W^T T = 0
