"""Gradient descent over a two-table star join whose entity table is kept in join order (ilargi_plan_cluster):
the one-pass iteration against the oracle's Alg. 1 and against the plan's unclustered iteration."""
import numpy as np
import pytest
import torch

import datagen
import oracle

pytestmark = pytest.mark.gpu

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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _run_gd(il, plan, model, y, lrs, iters, c_T):
    m = len(lrs)
    W = torch.zeros((c_T, m), device="cuda")
    lr = dev(np.asarray(lrs, dtype=np.float32))
    loss = torch.zeros(m, device="cuda")
    yd = y if isinstance(y, torch.Tensor) else dev(y)
    losses = []
    for _ in range(iters):
        il.ilargi_gd_step(plan, model, W, yd, lr, loss)
        losses.append(loss.cpu().numpy().copy())
    return W.cpu().numpy(), np.array(losses)


# (r_T, c_S, r_R, c_R, keys): the benchmark's shape scaled down; the narrowest tables; a full-width dimension table
# with a ragged last chunk; fan-out 1 with more rows of R than target rows and R the larger table (runs of more than
# eight rows of R per chunk, rows nobody joins); the same fan-out with R the smaller table (the usual sequence is
# kept); skewed keys (segments spanning many chunks); fewer rows than a chunk; one row of R
SHAPES = [(30_011, 20, 3_001, 200, "uniform"), (50_003, 4, 301, 24, "uniform"), (20_003, 8, 257, 256, "uniform"),
          (9_999, 4, 12_000, 24, "uniform"), (9_999, 32, 12_000, 4, "uniform"), (60_001, 12, 50, 36, ("zipf", 1.1)),
          (37, 16, 5, 8, "uniform"),
          (4_100, 28, 1, 12, "uniform")]


@pytest.mark.parametrize("model", ["linear", "logistic"])
@pytest.mark.parametrize("r_T,c_S,r_R,c_R,keys", SHAPES)
def test_gd_clustered_entity_table(il, model, r_T, c_S, r_R, c_R, keys):
    print(f"case {model} {r_T} {c_S} {r_R} {c_R} {keys}", flush=True)
    rng = datagen.rng_for(9100 + r_T + c_S + c_R)
    sch = datagen.star_schema(rng, r_T, c_S, [(r_R, c_R, keys)])
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=2)
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    lr = [0.05]
    W0, L0 = _run_gd(il, plan, code, y, lr, 5, sch.c_T)               # the plan's usual iteration
    il.ilargi_plan_cluster(plan)
    W, L = _run_gd(il, plan, code, y, lr, 5, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 1)), lr, 5)
    assert rel(W, W_ref) < GD_TOL
    assert np.abs(W - W_ref).max() <= GD_TOL * max(np.abs(W_ref).max(), 1e-30) * 10
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    assert rel(W, W0) < GD_TOL
    W2, L2 = _run_gd(il, plan, code, y, lr, 5, sch.c_T)
    assert np.array_equal(W, W2) and np.array_equal(L, L2)          # same bits on every run
    # the labels kept in join order with the copy: the same sums in the same order, so the same bits; another label
    # vector is gathered as before
    yd = dev(y)
    il.ilargi_plan_cluster(plan, y=yd)
    W4, L4 = _run_gd(il, plan, code, yd, lr, 5, sch.c_T)
    assert np.array_equal(W, W4) and np.array_equal(L, L4)
    y_other = (1.0 - y if model == "logistic" else -y).astype(np.float32)
    W5, L5 = _run_gd(il, plan, code, y_other, lr, 5, sch.c_T)
    W5_ref, L5_ref = oracle.gd(tg, model, y_other, np.zeros((sch.c_T, 1)), lr, 5)
    assert rel(W5, W5_ref) < GD_TOL
    np.testing.assert_allclose(L5, L5_ref, rtol=1e-4)
    # two models: the clustered copy is not used, the result is the usual one
    Wm, _ = _run_gd(il, plan, code, y, [0.05, 0.01], 2, sch.c_T)
    Wm_ref, _ = oracle.gd(tg, model, y, np.zeros((sch.c_T, 2)), [0.05, 0.01], 2)
    assert rel(Wm, Wm_ref) < GD_TOL
    # forgetting the copy brings back the usual iteration, bit for bit
    il.ilargi_plan_cluster(plan, None)
    W3, L3 = _run_gd(il, plan, code, y, lr, 5, sch.c_T)
    assert np.array_equal(W3, W0) and np.array_equal(L3, L0)


def test_clustered_copy_is_the_table_in_join_order(il):
    rng = datagen.rng_for(9200)
    sch = datagen.star_schema(rng, 7_001, 12, [(300, 16, "uniform")])
    srcs = il.schema_to_device(sch)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
    nbytes = il.ilargi_plan_cluster_bytes(plan)
    buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    il.ilargi_plan_cluster(plan, buf)
    torch.cuda.synchronize()
    fk = sch.sources[1].row_idx
    order = np.argsort(fk, kind="stable")
    raw = buf.cpu().numpy()
    sp = raw[:4 * sch.r_T * 12].view(np.float32).reshape(sch.r_T, 12)
    off = (4 * sch.r_T * 12 + 255) // 256 * 256
    keys = raw[off:off + 4 * sch.r_T].view(np.int32)
    assert np.array_equal(sp.view(np.uint32), sch.sources[0].D[order].view(np.uint32))
    assert np.array_equal(keys, fk[order])
    y = rng.standard_normal(sch.r_T).astype(np.float32)
    il.ilargi_plan_cluster(plan, buf, y=dev(y))
    torch.cuda.synchronize()
    off2 = off + (4 * sch.r_T + 255) // 256 * 256
    yp = buf.cpu().numpy()[off2:off2 + 4 * sch.r_T].view(np.float32)
    assert np.array_equal(yp.view(np.uint32), y[order].view(np.uint32))


def test_cluster_is_refused_where_it_does_not_apply(il):
    rng = datagen.rng_for(9300)
    # a key is missing: not every target row joins
    sch = datagen.star_schema(rng, 2_000, 8, [(100, 8, "uniform")])
    sch.sources[1].row_idx[17] = -1
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    with pytest.raises(il.IlargiError):
        il.ilargi_plan_cluster(plan)
    # three tables
    sch = datagen.star_schema(rng, 2_000, 8, [(100, 8, "uniform"), (50, 4, "uniform")])
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    with pytest.raises(il.IlargiError):
        il.ilargi_plan_cluster_bytes(plan)
    # an entity table whose rows are not whole float4s; a dimension table wider than 256 columns
    for c_S, c_R in [(6, 8), (8, 260)]:
        sch = datagen.star_schema(rng, 2_000, c_S, [(100, c_R, "uniform")])
        plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
        with pytest.raises(il.IlargiError):
            il.ilargi_plan_cluster(plan)
    # a buffer that is too small
    sch = datagen.star_schema(rng, 2_000, 8, [(100, 8, "uniform")])
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    small = torch.zeros(il.ilargi_plan_cluster_bytes(plan) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(il.IlargiError):
        il.ilargi_plan_cluster(plan, small)


def test_elementwise_in_place_on_the_entity_table_drops_the_copy(il):
    rng = datagen.rng_for(9400)
    sch = datagen.star_schema(rng, 6_000, 8, [(200, 12, "uniform")])
    srcs = il.schema_to_device(sch)
    plan = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=1)
    il.ilargi_plan_cluster(plan)
    il.ilargi_elementwise(plan, "mul", 0.5, outs=[D for D, _, _ in srcs])
    for s in sch.sources:
        s.D[...] = s.D * np.float32(0.5)
    tg = oracle.Target(sch)
    y = rng.standard_normal(sch.r_T).astype(np.float32)
    W, L = _run_gd(il, plan, il.LINEAR, y, [0.05], 3, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.05], 3)
    assert rel(W, W_ref) < GD_TOL


@pytest.mark.parametrize("r_T,c_S,r_R,c_R", [(30_011, 20, 3_001, 200), (20_003, 8, 257, 96), (9_000, 32, 1_000, 72)])
def test_crossprod_streams_the_clustered_copy(il, r_T, c_S, r_R, c_R):
    # the Gram matrix's pass over the entity table reads the join-ordered copy as a stream: the same sums in the same
    # order as with the rows gathered, so the same bits
    rng = datagen.rng_for(9500 + r_T)
    sch = datagen.star_schema(rng, r_T, c_S, [(r_R, c_R, "uniform")])
    tg = oracle.Target(sch)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    G0 = il.ilargi_crossprod(plan).cpu().numpy()
    il.ilargi_plan_cluster(plan)
    G1 = il.ilargi_crossprod(plan).cpu().numpy()
    assert np.array_equal(G0, G1)
    assert rel(G1, oracle.crossprod(tg)) < 1e-5
    assert np.array_equal(G1, G1.T)


@pytest.mark.parametrize("model", ["linear", "logistic"])
def test_gd_clustered_with_shared_dropped_and_unfed_columns(il, model):
    # the joined table listed first, a target column fed by both tables, one fed by nobody, one column of each
    # table dropped, rows of the joined table nobody uses; more than one chunk per wavefront
    rng = datagen.rng_for(9600)
    r_T, r_R = 200_003, 9_000
    S = rng.standard_normal((r_T, 8)).astype(np.float32)
    R = rng.standard_normal((r_R, 12)).astype(np.float32)
    fk = rng.integers(0, r_R // 2, size=r_T).astype(np.int32)
    r_map = np.array([9, 2, -1, 10, 12, 13, 14, 15, 16, 17, 18, 19], dtype=np.int32)
    s_map = np.array([0, 1, 2, 3, -1, 5, 6, 7], dtype=np.int32)
    sch = datagen.Schema([datagen.Source(R, fk, r_map), datagen.Source(S, None, s_map)], r_T, 21)
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels(model, oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(r_T))
    code = il.LINEAR if model == "linear" else il.LOGISTIC
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    yd = dev(y)
    il.ilargi_plan_cluster(plan, y=yd)
    W, L = _run_gd(il, plan, code, yd, [0.2], 6, sch.c_T)
    W_ref, L_ref = oracle.gd(tg, model, y, np.zeros((sch.c_T, 1)), [0.2], 6)
    assert rel(W, W_ref) < GD_TOL
    np.testing.assert_allclose(L, L_ref, rtol=1e-4)
    assert W[8, 0] == 0.0 and W[11, 0] == 0.0 and W[4, 0] == 0.0 and W[20, 0] == 0.0   # columns nobody feeds keep their weight
    il.ilargi_plan_cluster(plan, None)
    W0, L0 = _run_gd(il, plan, code, yd, [0.2], 6, sch.c_T)
    assert rel(W, W0) < GD_TOL


@pytest.mark.parametrize("prec", ["f32", "bf16"])
def test_wide_batch_streams_the_clustered_copy(il, prec):
    # many models at once: the join-order pass reads the join-ordered copy (and its labels) as streams -- the same
    # rows in the same order, so the same bits as with the rows gathered
    rng = datagen.rng_for(9700)
    sch = datagen.star_schema(rng, 40_003, 20, [(3_001, 72, "uniform")])
    tg = oracle.Target(sch)
    m = 40
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels("linear", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(sch.r_T))
    lrs = np.geomspace(1e-3, 5e-2, m)
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=m)
    precision = il.F32 if prec == "f32" else il.BF16_IN_F32_ACC
    yd, lr = dev(y), dev(lrs.astype(np.float32))

    def run():
        W = torch.zeros((sch.c_T, m), device="cuda")
        loss = torch.zeros(m, device="cuda")
        for _ in range(3):
            il.ilargi_gd_step(plan, il.LINEAR, W, yd, lr, loss, precision=precision)
        return W.cpu().numpy(), loss.cpu().numpy()

    W0, L0 = run()
    il.ilargi_plan_cluster(plan)                   # the copy without labels: labels gathered through the index
    W1, L1 = run()
    il.ilargi_plan_cluster(plan, y=yd)             # ... and with them
    W2, L2 = run()
    assert np.array_equal(W0, W1) and np.array_equal(L0, L1)
    assert np.array_equal(W0, W2) and np.array_equal(L0, L2)
    if prec == "f32":
        W_ref, _ = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, m)), lrs, 3)
        assert max(rel(W2[:, j], W_ref[:, j]) for j in range(m)) < GD_TOL


def test_clustered_iteration_replayed_from_a_captured_graph(il):
    # two iterations captured in a HIP graph (kernel launches only: nothing in the path clears memory with a memset
    # node) and replayed three times, with eager work and synchronisations between the replays: every replay
    # continues the same trajectory as eager calls, bit for bit
    rng = datagen.rng_for(9900)
    sch = datagen.star_schema(rng, 50_003, 12, [(2_000, 40, "uniform")])
    tg = oracle.Target(sch)
    w_star = rng.standard_normal(sch.c_T) / np.sqrt(sch.c_T)
    y = datagen.finish_labels("linear", oracle.lmm(tg, w_star.reshape(-1, 1)), 0.1 * rng.standard_normal(sch.r_T))
    plan = il.ilargi_plan_create(il.schema_to_device(sch), sch.r_T, sch.c_T, max_cx=1)
    yd, lr = dev(y), dev(np.array([0.1], dtype=np.float32))
    il.ilargi_plan_cluster(plan, y=yd)
    W_e = torch.zeros((sch.c_T, 1), device="cuda")
    loss_e = torch.zeros(1, device="cuda")
    eager = []
    for _ in range(6):
        il.ilargi_gd_step(plan, il.LINEAR, W_e, yd, lr, loss_e)
        eager.append((W_e.cpu().numpy().copy(), loss_e.cpu().numpy().copy()))
    W = torch.zeros((sch.c_T, 1), device="cuda")
    loss = torch.zeros(1, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        il.ilargi_gd_step(plan, il.LINEAR, W, yd, lr, loss)           # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    W.zero_()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(2):
            il.ilargi_gd_step(plan, il.LINEAR, W, yd, lr, loss)
    W.zero_()
    for k in range(3):
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(W.cpu().numpy(), eager[2 * k + 1][0])
        assert np.array_equal(loss.cpu().numpy(), eager[2 * k + 1][1])
        scratch = torch.randn(1 << 20, device="cuda").sum().item()      # eager work between the replays
        assert np.isfinite(scratch)
    W_ref, _ = oracle.gd(tg, "linear", y, np.zeros((sch.c_T, 1)), [0.1], 6)
    assert rel(W.cpu().numpy(), W_ref) < GD_TOL

