"""Host-side checks that need no GPU: the library loads, exports every symbol declared in
include/ra.h, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2409_10516_amd as ra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "ra.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ra_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"ra_build_index", "ra_decode_step", "ra_knn", "ra_project", "ra_search", "ra_attend",
            "ra_index_import", "ra_index_export", "ra_index_free", "ra_last_error"} <= set(names)
    L = ra.lib()
    for n in names:
        assert hasattr(L, n), n


def test_version_and_error_string():
    L = ra.lib()
    assert b"gfx950" in L.ra_version()
    assert isinstance(L.ra_last_error(), bytes)


def _fake():
    return C.c_void_p(0x1000)       # non-null; never dereferenced when validation fails first


@pytest.mark.parametrize("args,status,needle", [
    # K, Q, dt, n_seq, n_q, n_kv, N, M, d, knn
    ((None, _fake(), 1, 1, 4, 2, 100, 10, 128, 8), 1, "NULL"),
    ((_fake(), _fake(), 7, 1, 4, 2, 100, 10, 128, 8), 3, "dtype"),
    ((_fake(), _fake(), 1, 1, 4, 3, 100, 10, 128, 8), 1, "multiple"),
    ((_fake(), _fake(), 1, 1, 4, 2, 100, 10, 64, 8), 6, "d = 128"),
    ((_fake(), _fake(), 1, 1, 4, 2, 100, 10, 128, 101), 1, "exceeds N"),
    ((_fake(), _fake(), 1, 1, 4, 2, 100, 0, 128, 8), 1, "positive"),
    ((_fake(), _fake(), 1, 1, 4, 2, 1000, 10, 128, 65), 6, "RA_MAX_KNN"),
])
def test_knn_argument_validation(args, status, needle):
    L = ra.lib()
    out = _fake()
    rc = L.ra_knn(*args, None, out)
    assert rc == status
    assert needle in L.ra_last_error().decode()


def test_build_and_project_validation():
    L = ra.lib()
    h = C.c_void_p()
    assert L.ra_build_index(_fake(), _fake(), 1, 1, 4, 2, 100, 10, 128, 1, 8, None, C.byref(h)) == 1
    assert "deg" in L.ra_last_error().decode()
    assert L.ra_build_index(_fake(), _fake(), 1, 1, 4, 2, 100, 10, 128, 65, 8, None, C.byref(h)) == 6
    assert L.ra_project(_fake(), 0, 100, 10, 8, 8, None, _fake(), _fake()) == 1
    assert L.ra_project(None, 1, 100, 10, 8, 8, None, _fake(), _fake()) == 1


def test_decode_validation_without_index():
    L = ra.lib()
    rc = L.ra_decode_step(_fake(), None, _fake(), _fake(), 1, 100, 4, 8, 10, 20, 1, None, _fake(),
                          _fake(), None, None)
    assert rc == 1 and "handle" in L.ra_last_error().decode()
    assert L.ra_search(_fake(), None, _fake(), 1, 100, 4, 8, 10, 20, 1, None, _fake(), None) == 1
    # per-head budgets: the array is required, then the same checks as ra_decode_step
    rc = L.ra_decode_step_budgets(_fake(), None, _fake(), _fake(), 1, 100, 4, 8, 10, None, 20, 1, None,
                                  _fake(), _fake(), None, None)
    assert rc == 1 and "NULL" in L.ra_last_error().decode()
    rc = L.ra_decode_step_budgets(_fake(), None, _fake(), _fake(), 1, 100, 4, 8, 10, _fake(), 20, 1, None,
                                  _fake(), _fake(), None, None)
    assert rc == 1 and "handle" in L.ra_last_error().decode()
    assert L.ra_index_info(None, 0) == -1
    L.ra_index_free(None)            # must be a no-op


def test_settings_validation():
    """ra_index_configure / ra_test_configure reject a missing handle and unknown settings or values
    before anything touches a device; the process-wide test setting needs no handle."""
    L = ra.lib()
    L.ra_index_configure.restype = C.c_int
    L.ra_test_configure.restype = C.c_int
    assert L.ra_index_configure(None, 2, C.c_int64(64)) == 1 and "handle" in L.ra_last_error().decode()
    assert L.ra_test_configure(None, 101, C.c_int64(1)) == 1 and "handle" in L.ra_last_error().decode()
    assert L.ra_test_configure(None, 7, C.c_int64(0)) == 1 and "unknown" in L.ra_last_error().decode()
    assert L.ra_test_configure(None, 100, C.c_int64(9)) == 1
    assert L.ra_test_configure(None, 100, C.c_int64(2)) == 0
    assert L.ra_test_configure(None, 100, C.c_int64(0)) == 0


def test_import_validation():
    import numpy as np
    L = ra.lib()
    h = C.c_void_p()
    adj = np.full((1, 10, 4), -1, np.int32)
    ent = np.zeros(1, np.int32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    ent[0] = 10
    assert L.ra_index_import(p(adj), p(ent), 1, 1, 1, 10, 4, C.byref(h)) == 1
    assert "entry" in L.ra_last_error().decode()
    ent[0] = 0
    adj[0, 3, 2] = 10
    assert L.ra_index_import(p(adj), p(ent), 1, 1, 1, 10, 4, C.byref(h)) == 1
    assert "adjacency" in L.ra_last_error().decode()
    assert L.ra_index_import(p(adj), p(ent), 1, 1, 1, 10, 65, C.byref(h)) == 6


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(ValueError):
        ra.ra_knn(torch.zeros(1, 1, 8, 128), torch.zeros(1, 1, 4, 128), 2)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: --gpus 2 ends with a message and a non-zero status before anything
    touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
