"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported, and the
validation paths that run before any device work return the documented status codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2502_01985_amd as il

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ilargi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ilargi_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"ilargi_plan_create", "ilargi_lmm", "ilargi_tmm", "ilargi_crossprod", "ilargi_materialize",
            "ilargi_gd_step"} <= set(names)
    for name in names:
        assert hasattr(il.lib, name), name
    assert sorted(il.EXPORTED) == names


def test_version_and_error_string():
    assert il.ilargi_version() == "0.1"
    assert isinstance(il.ilargi_last_error(), str)


def _src(rows, cols, ident, cmap=None, dptr=4096, iptr=8192):
    cmap = np.arange(cols, dtype=np.int32) if cmap is None else np.asarray(cmap, dtype=np.int32)
    return (dptr, rows, cols, 0 if ident else iptr, cmap)


def test_workspace_bytes_grows_with_shapes():
    small = il.ilargi_plan_workspace_bytes([_src(1000, 4, True), _src(100, 8, False)], 1000, 12, 1)
    wide = il.ilargi_plan_workspace_bytes([_src(1000, 4, True), _src(100, 8, False)], 1000, 12, 16)
    tall = il.ilargi_plan_workspace_bytes([_src(100000, 4, True), _src(100, 8, False)], 100000, 12, 1)
    assert 0 < small < wide and small < tall
    assert small % 256 == 0
    # at least: inverse index (perm) and the residual buffer
    assert tall >= 4 * 100000 * 2


@pytest.mark.parametrize("kwargs,status", [
    (dict(n=0), il.ERR_SHAPE),
    (dict(n=17), il.ERR_SHAPE),
    (dict(r_T=-1), il.ERR_SHAPE),
    (dict(c_T=0), il.ERR_SHAPE),
    (dict(max_cx=0), il.ERR_SHAPE),
])
def test_workspace_bytes_rejects_bad_sizes(kwargs, status):
    args = dict(n=1, r_T=10, c_T=4, max_cx=1)
    args.update(kwargs)
    arr, keep = il.make_source_array([_src(10, 4, True)] * max(1, min(args["n"], 17)))
    out = ctypes.c_size_t(0)
    rc = il.lib.ilargi_plan_workspace_bytes(args["n"], arr, args["r_T"], args["c_T"], args["max_cx"], ctypes.byref(out))
    assert rc == status
    assert il.ilargi_last_error() != ""


def test_workspace_bytes_null_arguments():
    out = ctypes.c_size_t(0)
    assert il.lib.ilargi_plan_workspace_bytes(1, None, 10, 4, 1, ctypes.byref(out)) == il.ERR_NULL
    arr, keep = il.make_source_array([_src(10, 4, True)])
    assert il.lib.ilargi_plan_workspace_bytes(1, arr, 10, 4, 1, None) == il.ERR_NULL


def test_identity_source_needs_all_rows():
    arr, keep = il.make_source_array([_src(9, 4, True)])
    out = ctypes.c_size_t(0)
    assert il.lib.ilargi_plan_workspace_bytes(1, arr, 10, 4, 1, ctypes.byref(out)) == il.ERR_SHAPE


def _create(sources, r_T, c_T, workspace=256 * 1024, nbytes=1 << 40):
    arr, keep = il.make_source_array(sources)
    handle = ctypes.c_void_p(0)
    rc = il.lib.ilargi_plan_create(len(sources), arr, r_T, c_T, 1, workspace, nbytes, None, ctypes.byref(handle))
    return rc, handle


def test_plan_create_rejects_bad_column_maps_before_touching_the_device():
    rc, h = _create([_src(10, 3, True, cmap=[0, 1, 4])], 10, 4)
    assert rc == il.ERR_COLMAP and not h.value
    rc, h = _create([_src(10, 3, True, cmap=[0, -2, 1])], 10, 4)
    assert rc == il.ERR_COLMAP
    rc, h = _create([_src(10, 3, True, cmap=[2, 1, 2])], 10, 4)
    assert rc == il.ERR_COLMAP and "both map" in il.ilargi_last_error()
    # two different sources may share a target column; this one fails later, on the workspace
    rc, h = _create([_src(10, 2, True, cmap=[0, 1]), _src(10, 2, True, cmap=[1, 2])], 10, 4, nbytes=16)
    assert rc == il.ERR_WORKSPACE


def test_plan_create_rejects_null_and_misaligned_workspace():
    rc, _ = _create([_src(10, 4, True)], 10, 4, workspace=None)
    assert rc == il.ERR_NULL
    rc, _ = _create([_src(10, 4, True)], 10, 4, workspace=4096 + 8)
    assert rc == il.ERR_WORKSPACE
    rc, _ = _create([_src(10, 4, True, dptr=0)], 10, 4)
    assert rc == il.ERR_NULL
    arr, keep = il.make_source_array([_src(10, 4, True)])
    assert il.lib.ilargi_plan_create(1, arr, 10, 4, 1, 4096, 1 << 30, None, None) == il.ERR_NULL


def test_calls_reject_null_plan():
    assert il.lib.ilargi_lmm(None, 4096, 1, 4096, 0, None) == il.ERR_NULL
    assert il.lib.ilargi_tmm(None, 4096, 1, 4096, 0, None) == il.ERR_NULL
    assert il.lib.ilargi_crossprod(None, 4096, None) == il.ERR_NULL
    assert il.lib.ilargi_materialize(None, 4096, None) == il.ERR_NULL
    assert il.lib.ilargi_gd_step(None, 0, 4096, 1, 4096, 4096, None, 0, None) == il.ERR_NULL
    assert il.lib.ilargi_plan_destroy(None) == il.ERR_NULL


# ----------------------------------------------------------------------------- ilargi_choose (host only)
def _shapes(sch):
    return [(s.D.shape[0], s.D.shape[1], s.row_idx is not None) for s in sch.sources]


def test_choose_reports_the_paper_formulas():
    import datagen
    import oracle
    for sch in (datagen.config0(), datagen.star_schema(datagen.rng_for(3), 5_000, 7, [(40, 30, "uniform"), (900, 3, "uniform")])):
        c = il.ilargi_choose(_shapes(sch), sch.r_T, sch.c_T)
        o_mat, o_fact = oracle.complexity_lr(sch)
        assert c["complexity_ratio"] == pytest.approx(o_mat / o_fact, rel=1e-12)
        tr, fr = oracle.tuple_and_feature_ratio(sch)
        assert c["tuple_ratio"] == pytest.approx(tr, rel=1e-12) and c["feature_ratio"] == pytest.approx(fr, rel=1e-12)
        assert c["morpheus_rule"] == int(tr >= 5.0 and fr >= 1.0)


def test_choose_decision_follows_its_byte_model():
    # wide dimension table, many target rows per dimension row: factorize; feature ratio 1/4: materialize
    star = [(1_000_000, 20, False), (10_000, 800, True)]
    cs = il.ilargi_choose(star, 1_000_000, 820)
    assert cs["factorize"] == 1 and cs["bytes_factorized"] < cs["bytes_materialized"] / 5
    thin = [(1_000_000, 40, False), (500_000, 10, True)]
    c = il.ilargi_choose(thin, 1_000_000, 50)
    assert c["factorize"] == 0 and c["seconds_materialized"] < c["seconds_factorized"]
    # the join is paid once: a single iteration never repays it when the per-iteration times are close
    few = il.ilargi_choose(thin, 1_000_000, 50, iterations=1)
    assert few["factorize"] == 1 and few["bytes_join"] > few["bytes_materialized"] * 0.9
    # tiny tables are decided by launches: a two-table star join with short rows runs an iteration as one launch
    # against two for its joined table (whose 12-column rows are too many for the single-launch form) ...
    tiny = il.ilargi_choose([(10_000, 4, False), (1_000, 8, True)], 10_000, 12)
    assert tiny["factorize"] == 1
    # ... while a tiny schema outside that form takes its several dependent launches against two
    tiny3 = il.ilargi_choose([(10_000, 4, False), (1_000, 8, True), (500, 4, True)], 10_000, 16)
    assert tiny3["factorize"] == 0
    # a small schema with a wide dimension table moves fewer bytes factorized but needs more launches: the
    # launch price decides
    small = [(10_000, 4, False), (100, 64, True)]
    assert il.ilargi_choose(small, 10_000, 68)["factorize"] == 0
    free = il.ilargi_choose(small, 10_000, 68, launch_seconds=1e-9)
    assert free["factorize"] == 1 and free["bytes_factorized"] < free["bytes_materialized"]
    # tables wider than 256 columns are read twice per iteration (no shared pass)
    wide = il.ilargi_choose([(1_000, 300, False)], 1_000, 300)
    narrow = il.ilargi_choose([(1_000, 200, False)], 1_000, 200)
    assert wide["bytes_materialized"] / narrow["bytes_materialized"] > 2.9
    # more models in a pass move more operand bytes but the same tables
    m4 = il.ilargi_choose(star, 1_000_000, 820, models=4)
    assert m4["bytes_factorized"] > cs["bytes_factorized"] and m4["factorize"] == 1
    # stacked tables (the identity source ends before the target does): one model reads every table once per
    # iteration, which is fewer bytes than the joined table with its shared columns stored once per row ...
    union = [(2_000_000, 64, False), (2_000_000, 64, True)]
    u1 = il.ilargi_choose(union, 3_400_000, 96)
    assert u1["factorize"] == 1 and u1["bytes_factorized"] == pytest.approx(4.0 * 2 * 2_000_000 * 64, rel=0.05)
    assert u1["bytes_factorized"] < 0.85 * u1["bytes_materialized"]
    # ... while two models at once go through the factorized sequence, which reads the second table twice
    u2 = il.ilargi_choose(union, 3_400_000, 96, models=2)
    assert u2["bytes_factorized"] > 1.4 * u1["bytes_factorized"] and u2["factorize"] == 0
    # rows wider than the on-the-fly join takes: the sequence again
    u3 = il.ilargi_choose([(2_000_000, 128, False), (2_000_000, 128, True)], 3_400_000, 192)
    assert u3["bytes_factorized"] > 1.4 * 4.0 * 2 * 2_000_000 * 128


def test_choose_rejects_bad_arguments():
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_choose([(10, 2, False)], 10, 2, iterations=0)
    assert ei.value.status == il.ERR_SHAPE
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_choose([(10, 2, False)], 10, 0)
    assert ei.value.status == il.ERR_SHAPE


# ----------------------------------------------------------------------------- sparse sources (host side)
def test_workspace_grows_with_the_stored_entries_of_a_sparse_source():
    cm = np.arange(8, dtype=np.int32)
    none = il.ilargi_plan_workspace_bytes([(0, 1000, 8, 0, cm, 1, 1, 1, 0)], 1000, 8, 1)
    sparse = il.ilargi_plan_workspace_bytes([(0, 1000, 8, 0, cm, 1, 1, 1, 4000)], 1000, 8, 1)
    more = il.ilargi_plan_workspace_bytes([(0, 1000, 8, 0, cm, 1, 1, 1, 8000)], 1000, 8, 1)
    # column-sorted rows and values and two temporaries: at least 16 bytes per stored entry, sort buffers on top
    assert sparse - none >= 16 * 4000 and more - sparse >= 16 * 4000
    with pytest.raises(il.IlargiError) as ei:
        il.ilargi_plan_workspace_bytes([(0, 1000, 8, 0, cm, 1, 1, 1, 8001)], 1000, 8, 1)    # more entries than cells
    assert ei.value.status == il.ERR_SHAPE


def test_choose_counts_stored_entries_for_sparse_tables():
    dense = il.ilargi_choose([(100_000, 20, False), (10_000, 200, True)], 100_000, 220)
    sparse = il.ilargi_choose([(100_000, 20, False, 200_000), (10_000, 200, True, 200_000)], 100_000, 220)
    # Tab. 2: the factorized cost is counted in non-zero elements
    assert sparse["complexity_ratio"] > dense["complexity_ratio"]
    assert sparse["bytes_factorized"] < dense["bytes_factorized"]
