"""ilargi_plan_create_static (the plan lives in the library's static scratch array, no device allocation)
against ilargi_plan_create (caller's workspace): same inverse indices, same operator results, on two plans in
a row, the second over a smaller input so that the array still holds the first plan's data."""
import gc

import numpy as np
import pytest

import datagen
import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def il():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_01985_amd as mod
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (nb if nb > 0 else 1.0))


def _same_bits(a, b):
    return np.array_equal(a.cpu().numpy().view(np.uint32), b.cpu().numpy().view(np.uint32))


def _compare(il, sch, seed, max_cx=16):
    """Runs every hot-path operator on a plan in the caller's workspace and on one in the static array."""
    srcs = il.schema_to_device(sch)
    ref = il.ilargi_plan_create(srcs, sch.r_T, sch.c_T, max_cx=max_cx)
    # tensors of earlier tests that are still waiting for the garbage collector must not be released in between
    gc.collect()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = il.ilargi_plan_create_static(srcs, sch.r_T, sch.c_T, max_cx=max_cx)
    assert torch.cuda.memory_allocated() <= before, "creating the static plan allocated device memory"
    assert st.workspace is None
    try:
        # integer work: the inverse indices are identical
        for k, s in enumerate(sch.sources):
            rp_a, pm_a = il.ilargi_plan_inverse_index(ref, k)
            rp_b, pm_b = il.ilargi_plan_inverse_index(st, k)
            if rp_a is None:
                assert rp_b is None
                continue
            assert np.array_equal(rp_a, rp_b) and np.array_equal(pm_a, pm_b), f"inverse index of source {k}"
        assert _same_bits(il.ilargi_materialize(ref), il.ilargi_materialize(st))
        tg = oracle.Target(sch)
        rng = datagen.rng_for(seed)
        for cx in (1, 3, max_cx):
            X = rng.standard_normal((sch.c_T, cx)).astype(np.float32)
            Y = rng.standard_normal((sch.r_T, cx)).astype(np.float32)
            a, b = il.ilargi_lmm(ref, dev(X)), il.ilargi_lmm(st, dev(X))
            assert rel(b.cpu().numpy(), a.cpu().numpy()) < 1e-6 and rel(b.cpu().numpy(), oracle.lmm(tg, X)) < 1e-5
            assert _same_bits(a, b), f"lmm cx={cx}"
            a, b = il.ilargi_tmm(ref, dev(Y)), il.ilargi_tmm(st, dev(Y))
            assert rel(b.cpu().numpy(), a.cpu().numpy()) < 1e-6 and rel(b.cpu().numpy(), oracle.tmm(tg, Y)) < 1e-5
            assert _same_bits(a, b), f"tmm cx={cx}"
        a, b = il.ilargi_crossprod(ref), il.ilargi_crossprod(st)
        assert rel(b.cpu().numpy(), oracle.crossprod(tg)) < 1e-5
        assert _same_bits(a, b), "crossprod"
        # three iterations of Alg. 1 from the same start
        y = dev(rng.standard_normal(sch.r_T).astype(np.float32))
        lr = dev(np.array([0.05], dtype=np.float32))
        Wa = torch.zeros((sch.c_T, 1), device="cuda")
        Wb = torch.zeros((sch.c_T, 1), device="cuda")
        la, lb = torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
        for _ in range(3):
            il.ilargi_gd_step(ref, il.LINEAR, Wa, y, lr, la)
            il.ilargi_gd_step(st, il.LINEAR, Wb, y, lr, lb)
        assert rel(Wb.cpu().numpy(), Wa.cpu().numpy()) < 1e-6
        assert _same_bits(Wa, Wb) and _same_bits(la, lb), "gd_step"
        torch.cuda.synchronize()
    finally:
        torch.cuda.synchronize()
        st.destroy()
        ref.destroy()


def test_static_plan_matches_workspace_plan_twice_in_a_row_second_smaller(il):
    assert il.ilargi_static_scratch_bytes() == 128 << 20
    big = datagen.config1(r_S=30_011, r_R=3_001, c_R=200)          # several tiles, ragged tails
    small = datagen.config2(r_S=5_003, dim_rows=(400, 200, 40))    # smaller, three joined tables, a long segment
    _compare(il, big, 901)
    _compare(il, small, 902)


def test_static_plan_limits(il):
    sch = datagen.config0()
    srcs = il.schema_to_device(sch)
    first = il.ilargi_plan_create_static(srcs, sch.r_T, sch.c_T, max_cx=1)
    try:
        # one static plan per device at a time
        with pytest.raises(il.IlargiError) as e:
            il.ilargi_plan_create_static(srcs, sch.r_T, sch.c_T, max_cx=1)
        assert e.value.status == il.ERR_WORKSPACE and "live plan" in str(e.value)
    finally:
        torch.cuda.synchronize()
        first.destroy()
    # a plan beyond the array's size is refused before any device work, and leaves the array free
    need = il.ilargi_plan_workspace_bytes([(1, s.D.shape[0], s.D.shape[1], 0 if s.row_idx is None else 1, s.col_map)
                                           for s in sch.sources], sch.r_T, sch.c_T, 4096)
    assert need > il.ilargi_static_scratch_bytes()
    with pytest.raises(il.IlargiError) as e:
        il.ilargi_plan_create_static(srcs, sch.r_T, sch.c_T, max_cx=4096)
    assert e.value.status == il.ERR_WORKSPACE and "static scratch" in str(e.value)
    again = il.ilargi_plan_create_static(srcs, sch.r_T, sch.c_T, max_cx=1)
    X = dev(np.ones((sch.c_T, 1), dtype=np.float32))
    got = il.ilargi_lmm(again, X).cpu().numpy()
    assert rel(got, oracle.lmm(oracle.Target(sch), np.ones((sch.c_T, 1), dtype=np.float32))) < 1e-5
    torch.cuda.synchronize()
    again.destroy()
