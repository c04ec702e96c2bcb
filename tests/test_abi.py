"""The C-ABI library loads and exports every symbol include/metis.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "metis.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(metis_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    from paper_2509_00404_amd import metis
    assert _declared() == metis.exported_symbols()


def test_library_exports_every_declared_symbol():
    from paper_2509_00404_amd import metis
    if not os.path.exists(metis.LIB_PATH):
        pytest.skip("library not built (run __graft_entry__.build())")
    L = ctypes.CDLL(metis.LIB_PATH)
    for name in _declared():
        assert hasattr(L, name), name
    assert metis.lib().metis_version() >= 1
    assert metis.lib().metis_status_string(-2) == b"bad shape"


def test_host_side_argument_checks_need_no_gpu():
    from paper_2509_00404_amd import metis
    if not os.path.exists(metis.LIB_PATH):
        pytest.skip("library not built")
    L = metis.lib()
    assert L.metis_sample_count(8192, 64, 16, 1.0 / 16) == 512
    assert L.metis_sample_count(256, 8, 8, 0.25) == 64
    assert L.metis_sample_count(8192, 64, 16, 0.001) == 80
    assert L.metis_sample_count(50, 64, 16, 1.0) == 50
    assert L.metis_sample_count(100, 4, 4, 0.0) == 0
    # null pointers and bad shapes are refused before anything is enqueued
    assert L.metis_sample_rows(None, 1, 100, 10, None) == -1
    assert L.metis_gaussian_omega(None, 1, 0, 4, None) == -1
    assert L.metis_quantize(None, None, None, None) == -1
    assert L.metis_quantize_sr(None, None, 0, None, None) == -1


def test_tensor_scale_helper_is_the_smallest_covering_power_of_two():
    from paper_2509_00404_amd import metis
    if not os.path.exists(metis.LIB_PATH):
        pytest.skip("library not built")
    import numpy as np
    ts = metis.tensor_scale
    assert ts(6 * 448.0) == 1.0 and ts(6 * 448.0 + 1) == 2.0 and ts(1.0) == 2.0 ** -11
    assert ts(0.0) == 1.0 and ts(-3.0) == 1.0 and ts(float("inf")) == 1.0 and ts(float("nan")) == 1.0
    rs = np.random.default_rng(0)
    for a in np.exp(rs.uniform(-40, 40, 2000)).astype(np.float32):
        g = ts(float(a))
        m, e = np.frexp(g)
        assert m == 0.5                                            # a power of two
        assert 2688.0 * g >= float(a) and 2688.0 * (g / 2) < float(a)


def test_bench_refuses_more_than_one_gpu():
    """One GPU is the whole target: `bench.py --gpus N` with N > 1 exits with a message before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""
