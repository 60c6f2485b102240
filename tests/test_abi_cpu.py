"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and
reports argument errors before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_18856_amd import bsse

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bsse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bsse_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = bsse.lib()
    names = _declared_symbols()
    assert "bsse_create" in names and "bsse_sweep" in names and "bsse_lattice" in names
    for name in names:
        assert hasattr(L, name), name
    assert sorted(bsse.EXPORTS) == names


def _tiny():
    A = np.arange(18, dtype=np.float32).reshape(2, 3, 3)
    B = A[::-1].copy()
    p = np.array([0.7, 0.3], np.float32)
    return A, B, p


def _status(fn, *a, **k):
    with pytest.raises(bsse.BsseError) as e:
        fn(*a, **k)
    return e.value.status


def test_create_argument_errors_come_before_any_device_call():
    A, B, p = _tiny()
    L = bsse.lib()
    h = ctypes.c_void_p()
    opt = bsse.bsse_options(0, 0, -1)
    bad = [
        (0, 3, 2), (3, 0, 2), (3, 3, 0), (-1, 3, 2), (5000, 3, 2), (3, 70000, 2),
    ]
    for (m, n, K) in bad:
        st = L.bsse_create_ex(m, n, K, A.ctypes.data, B.ctypes.data, p.ctypes.data,
                              ctypes.byref(opt), ctypes.byref(h))
        assert st == bsse.BSSE_EINVAL and not h.value
        assert bsse.bsse_last_error()
    assert L.bsse_create_ex(3, 3, 2, None, B.ctypes.data, p.ctypes.data, ctypes.byref(opt),
                            ctypes.byref(h)) == bsse.BSSE_EINVAL
    assert L.bsse_create_ex(3, 3, 2, A.ctypes.data, B.ctypes.data, p.ctypes.data, None,
                            ctypes.byref(h)) == bsse.BSSE_EINVAL
    assert L.bsse_create_ex(3, 3, 2, A.ctypes.data, B.ctypes.data, p.ctypes.data,
                            ctypes.byref(opt), None) == bsse.BSSE_EINVAL
    for o in (bsse.bsse_options(7, 0, -1), bsse.bsse_options(0, 9, -1), bsse.bsse_options(0, 0, -5)):
        assert L.bsse_create_ex(3, 3, 2, A.ctypes.data, B.ctypes.data, p.ctypes.data,
                                ctypes.byref(o), ctypes.byref(h)) == bsse.BSSE_EINVAL
    # too many payoff entries
    assert L.bsse_create_ex(4096, 65535, 2, A.ctypes.data, B.ctypes.data, p.ctypes.data,
                            ctypes.byref(opt), ctypes.byref(h)) == bsse.BSSE_EINVAL
    # non-finite payoffs and priors
    A2 = A.copy(); A2[1, 2, 0] = np.nan
    assert _status(bsse.bsse_create, 3, 3, 2, A2, B, p) == bsse.BSSE_ENOTFINITE
    B2 = B.copy(); B2[0, 0, 1] = np.inf
    assert _status(bsse.bsse_create, 3, 3, 2, A, B2, p) == bsse.BSSE_ENOTFINITE
    assert _status(bsse.bsse_create, 3, 3, 2, A, B, np.array([np.nan, 1], np.float32)) == bsse.BSSE_ENOTFINITE
    # prior off the simplex
    assert _status(bsse.bsse_create, 3, 3, 2, A, B, np.array([0.7, 0.2], np.float32)) == bsse.BSSE_EINVAL
    assert _status(bsse.bsse_create, 3, 3, 2, A, B, np.array([1.5, -0.5], np.float32)) == bsse.BSSE_EINVAL
    # a shape with no matrix-core path cannot be forced onto it
    assert _status(bsse.bsse_create, 3, 3, 2, A, B, p, path=bsse.BSSE_PATH_MFMA) == bsse.BSSE_EINVAL


def test_null_handles_are_rejected():
    L = bsse.lib()
    res = bsse.bsse_result()
    c = ctypes.c_int64()
    assert L.bsse_sweep(None, None, 0, ctypes.byref(res), None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_chunk(None, None, 0, 0) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_result(None, ctypes.byref(res), None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_reset(None) == bsse.BSSE_EINVAL
    assert L.bsse_lattice(None, 4, ctypes.byref(c)) == bsse.BSSE_EINVAL
    assert L.bsse_dirichlet(None, 1, 0, 4, None) == bsse.BSSE_EINVAL
    assert L.bsse_eval(None, None, 0, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_priors(None, None, 0, None, 1, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_topk(None, None, 0, 1, None, None, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_lattice_around(None, 4, None, 0.5, ctypes.byref(c)) == bsse.BSSE_EINVAL
    assert L.bsse_refine(None, 1, 1, 4, 0, 0, 0.5, 0.5, None, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_solve_realised(None, None, 0, 1, None, None, None, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_dirichlet_around(None, 1, 0, 4, None, 0.5, None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_dirichlet(None, 1, 0, 4, ctypes.byref(res), None) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_dirichlet_chunk(None, 1, 0, 4, 0) == bsse.BSSE_EINVAL
    assert L.bsse_sweep_best_row(None, None) == bsse.BSSE_EINVAL
    assert L.bsse_set_stream(None, None) == bsse.BSSE_EINVAL
    assert L.bsse_set_timing(None, 1) == bsse.BSSE_EINVAL
    L.bsse_destroy(None)
    assert bsse.lib().bsse_path_name(None) == b""


def test_ceiling_measurements_check_their_arguments_first():
    L = bsse.lib()
    d = ctypes.c_double()
    assert L.bsse_measure_ceilings(-1, None, None, None, None) == bsse.BSSE_EINVAL
    assert L.bsse_measure_ceilings(-2, ctypes.byref(d), ctypes.byref(d), ctypes.byref(d), ctypes.byref(d)) == bsse.BSSE_EINVAL
    assert L.bsse_measure_mixed_ceiling(-1, 32, 312, None) == bsse.BSSE_EINVAL
    assert L.bsse_measure_mixed_ceiling(-2, 32, 312, ctypes.byref(d)) == bsse.BSSE_EINVAL
    for mf, va in [(0, 24), (3, 24), (4100, 24), (32, -24), (32, 30), (32, 65544)]:
        assert L.bsse_measure_mixed_ceiling(-1, mf, va, ctypes.byref(d)) == bsse.BSSE_EINVAL


def test_lattice_count_on_host():
    from math import comb
    for m, N in [(3, 100), (1, 9), (2, 1), (8, 12), (32, 6), (4, 1000)]:
        assert bsse.bsse_lattice_count(m, N) == comb(N + m - 1, m - 1)
    assert bsse.bsse_lattice_count(3, 100) == 5151
    assert _status(bsse.bsse_lattice_count, 32, 1000) == bsse.BSSE_EOVERFLOW
    assert _status(bsse.bsse_lattice_count, 128, 128) == bsse.BSSE_EOVERFLOW
    assert _status(bsse.bsse_lattice_count, 3, 0) == bsse.BSSE_EINVAL
    assert _status(bsse.bsse_lattice_count, 0, 5) == bsse.BSSE_EINVAL
    assert "2^40" in bsse.bsse_last_error() or bsse.bsse_last_error()


def test_status_names():
    assert bsse.status_name(0) == "BSSE_OK"
    assert bsse.status_name(bsse.BSSE_EOVERFLOW) == "BSSE_EOVERFLOW"


def test_valid_create_without_a_device_reports_edevice():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    A, B, p = _tiny()
    assert _status(bsse.bsse_create, 3, 3, 2, A, B, p) == bsse.BSSE_EDEVICE


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: --gpus 2 exits with a message before touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
