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
