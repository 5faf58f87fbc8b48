"""Boundary checks that need no GPU: the C-ABI library loads, exports every function that
include/exat.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2311_13693_amd import exat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "exat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(exat_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = _declared()
    assert len(names) >= 9
    L = exat.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(exat.EXPORTS) == names


def test_strerror_is_total():
    for s in range(-8, 2):
        assert isinstance(exat.strerror(s), str) and exat.strerror(s)
    assert exat.strerror(0) == "success"


def _desc(**kw):
    base = dict(I=8, J=8, K=8, L=2, M=2, N=2, P=1, dI=4, dJ=4, dK=4, in_dtype=0)
    base.update(kw)
    return exat.make_desc(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(I=0), exat.ERR_SHAPE), (dict(J=-3), exat.ERR_SHAPE), (dict(K=2 ** 31), exat.ERR_SHAPE),
    (dict(L=0), exat.ERR_SHAPE), (dict(M=65), exat.ERR_SHAPE), (dict(P=0), exat.ERR_SHAPE),
    (dict(dI=9), exat.ERR_SHAPE), (dict(dJ=0), exat.ERR_SHAPE), (dict(dK=16), exat.ERR_SHAPE),
    (dict(in_dtype=7), exat.ERR_DTYPE), (dict(P=2 ** 20, L=64), exat.ERR_SHAPE),
])
def test_plan_create_rejects_bad_descriptors(kw, code):
    h = ctypes.c_void_p()
    d = _desc(**kw)
    assert exat.lib().exat_plan_create(ctypes.byref(h), ctypes.byref(d)) == code
    assert not h


def test_null_arguments_are_errors_not_crashes():
    L = exat.lib()
    d = _desc()
    h = ctypes.c_void_p()
    assert L.exat_plan_create(None, ctypes.byref(d)) == exat.ERR_NULL
    assert L.exat_plan_create(ctypes.byref(h), None) == exat.ERR_NULL
    assert L.exat_plan_destroy(None) == exat.OK
    assert L.exat_set_factors(None, None, 0, None, 0, None, 0, None) == exat.ERR_NULL
    assert L.exat_compress(None, None, None, None) == exat.ERR_NULL
    assert L.exat_compress_block(None, None, 0, 0, 0, None) == exat.ERR_NULL
    assert L.exat_finalize(None, None, None) == exat.ERR_NULL
    assert L.exat_compress_gen(None, None, None, None, None) == exat.ERR_NULL
    g = exat.Gen(None, None, None, 3, 1, 0.0)
    assert L.exat_gen_block(ctypes.byref(d), ctypes.byref(g), 0, 0, 0, None, None) == exat.ERR_NULL
    assert L.exat_gen_block(None, ctypes.byref(g), 0, 0, 0, None, None) == exat.ERR_NULL
    g2 = exat.Gen(1, 1, 1, 0, 1, 0.0)   # R = 0 (pointers are never dereferenced on this path)
    assert L.exat_gen_block(ctypes.byref(d), ctypes.byref(g2), 0, 0, 0, ctypes.c_void_p(1), None) == exat.ERR_SHAPE
    g3 = exat.Gen(1, 1, 1, 2, 1, 0.0)
    assert L.exat_gen_block(ctypes.byref(d), ctypes.byref(g3), 2, 0, 0, ctypes.c_void_p(1), None) == exat.ERR_SHAPE


def test_stage1_argument_errors():
    # validation happens before the first HIP call, so this runs without a GPU
    L = exat.lib()
    h = ctypes.c_void_p()
    rp = np.array([0, 1, 2], dtype=np.int64); ci = np.array([0, 1], dtype=np.int32); v = np.ones(2, dtype=np.float32)
    good = exat.make_csr(rp, ci, v, 4)
    for bad, code in ((exat.make_csr(rp, ci, v, 5), exat.ERR_SHAPE),                                  # cols != I
                      (exat.make_csr(rp, np.array([0, 4], dtype=np.int32), v, 4), exat.ERR_SHAPE),    # column out of range
                      (exat.make_csr(np.array([0, 2, 1], dtype=np.int64), ci, v, 4), exat.ERR_SHAPE),  # decreasing rowptr
                      (exat.make_csr(np.zeros(130, dtype=np.int64), ci[:0], v[:0], 4), exat.ERR_SHAPE)):  # 129 rows
        assert L.exat_stage1_create(ctypes.byref(h), 4, 4, 4, ctypes.byref(bad), ctypes.byref(good), ctypes.byref(good)) == code
    assert L.exat_stage1_create(ctypes.byref(h), 4, 4, 4, None, ctypes.byref(good), ctypes.byref(good)) == exat.ERR_NULL
    assert L.exat_stage1_create(ctypes.byref(h), 0, 4, 4, ctypes.byref(good), ctypes.byref(good), ctypes.byref(good)) == exat.ERR_SHAPE
    assert L.exat_stage1_apply(None, None, None, None) == exat.ERR_NULL
    assert L.exat_stage1_destroy(None) == exat.OK


def test_cpals_argument_errors():
    # validation happens before the first HIP call; the non-null pointers are never dereferenced
    L = exat.lib()
    p = ctypes.c_void_p(256)
    assert L.exat_cpals(None, 2, 2, 2, 1, 1, 1, p, p, p, p, None) == exat.ERR_NULL
    assert L.exat_cpals(p, 2, 2, 2, 1, 1, 1, p, p, p, None, None) == exat.ERR_NULL
    assert L.exat_cpals(p, 65, 2, 2, 1, 1, 1, p, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_cpals(p, 2, 2, 2, 1, 65, 1, p, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_cpals(p, 2, 2, 2, 0, 1, 1, p, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_cpals(p, 2, 2, 2, 1, 1, -1, p, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_cpals_workspace_floats(3, 4, 5, 6) >= 2 * 3 * 4 * 5 * 6      # two copies of Y plus partial results
    assert L.exat_cpals_workspace_floats(0, 4, 5, 6) == 0


def test_ls_argument_errors():
    # validation happens before the first HIP call; the non-null pointers are never dereferenced
    L = exat.lib()
    p = ctypes.c_void_p(256)
    ld = ctypes.c_int64(8)
    tol = ctypes.c_float(1e-6)
    assert L.exat_ls(None, ld, 2, 4, 8, p, 2, 1, tol, p, p, p, None) == exat.ERR_NULL
    assert L.exat_ls(p, ld, 2, 4, 8, p, 2, 1, tol, p, None, None, None) == exat.ERR_NULL     # relres may be NULL, work not
    assert L.exat_ls(p, ctypes.c_int64(7), 2, 4, 8, p, 2, 1, tol, p, p, p, None) == exat.ERR_SHAPE   # ldU < I
    assert L.exat_ls(p, ld, 2, 4, 8, p, 65, 1, tol, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_ls(p, ld, 0, 4, 8, p, 2, 1, tol, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_ls(p, ld, 2, 4, 8, p, 2, -1, tol, p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_ls(p, ld, 2, 4, 8, p, 2, 1, ctypes.c_float(-1.0), p, p, p, None) == exat.ERR_SHAPE
    assert L.exat_ls_workspace_floats(2, 4, 8, 2) >= 4 * 8 * 2 + 3 * 8 * 2
    assert L.exat_ls_workspace_floats(2, 4, 8, 65) == 0


def test_timing_argument_errors():
    L = exat.lib()
    f = ctypes.c_float()
    assert L.exat_plan_timing_of(None, 0, ctypes.byref(f), ctypes.byref(f)) == exat.ERR_NULL
    assert L.exat_plan_last_timing(None, ctypes.byref(f), ctypes.byref(f)) == exat.ERR_NULL


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU only: any other --gpus value exits with status 2 and says why, before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
