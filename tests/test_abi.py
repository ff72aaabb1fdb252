"""CPU-only checks of the C ABI: the library loads, exports every function the header declares, reports bad
arguments instead of crashing, and its host-only closed forms agree with the oracle's."""
from __future__ import annotations

import ctypes
import math
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvfuse.h")
LIB = os.path.join(ROOT, "paper_2601_03067_amd", "libkvfuse.so")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvfuse_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2601_03067_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_every_declared_function_is_exported(lib):
    names = _declared()
    assert len(names) >= 25 and "kvfuse_similarity" in names and "kvfuse_paged_decode_attn_shared" in names
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, f"declared in include/kvfuse.h but not exported: {missing}"


def test_null_arguments_are_errors_not_crashes(lib):
    lib.kvfuse_last_error.restype = ctypes.c_char_p
    assert lib.kvfuse_create(None, 0, None) != 0
    assert lib.kvfuse_block_norms(None, None, None) != 0
    assert lib.kvfuse_fuse_tree(None, None, ctypes.c_double(0.9), ctypes.c_double(1e-3), None, None, None, None, 0) != 0
    assert lib.kvfuse_paged_decode_attn_shared(None, None, None, None, None, ctypes.c_float(1.0), None) != 0
    assert lib.kvfuse_pair_cosines(None, None, None, None, 0, None) != 0
    assert lib.kvfuse_predict_compression(None, 0, ctypes.c_double(1.0), None, None) != 0
    assert lib.kvfuse_last_error(None) == b"null context"
    out = ctypes.c_size_t(0)
    assert lib.kvfuse_decode_workspace_bytes(-1, 1, 4, 1, 128, 1, ctypes.byref(out)) != 0
    assert lib.kvfuse_decode_workspace_bytes(2, 3, 8, 2, 128, 40, ctypes.byref(out)) == 0 and out.value >= 256


def test_threshold_closed_forms_match_the_oracle(lib):
    from oracle import threshold as th
    f64 = ctypes.c_double
    lib.kvfuse_exceedance_rate.restype = f64
    lib.kvfuse_exceedance_rate.argtypes = [f64] * 4
    lib.kvfuse_threshold_for_rate.restype = f64
    lib.kvfuse_threshold_for_rate.argtypes = [f64] * 4
    lib.kvfuse_threshold_feedback.restype = f64
    lib.kvfuse_threshold_feedback.argtypes = [f64] * 6
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = float(rng.integers(10, 10_000_000))
        mu, sigma = float(rng.uniform(-0.2, 0.6)), float(rng.uniform(1e-3, 0.3))
        u = float(rng.uniform(mu - 3 * sigma, mu + 6 * sigma))
        want = th.exceedance_rate(n, mu, sigma, u)
        got = lib.kvfuse_exceedance_rate(n, mu, sigma, u)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-300)
        if 1e-9 * n < want < 0.999 * n:
            assert lib.kvfuse_threshold_for_rate(n, mu, sigma, want) == pytest.approx(th.threshold_for_rate(n, mu, sigma, want), abs=1e-9)
            assert lib.kvfuse_threshold_for_rate(n, mu, sigma, want) == pytest.approx(u, abs=1e-9)
    assert lib.kvfuse_exceedance_rate(100.0, 0.5, 0.0, 0.4) == 100.0 and lib.kvfuse_exceedance_rate(100.0, 0.3, 0.0, 0.4) == 0.0
    assert math.isnan(lib.kvfuse_threshold_for_rate(100.0, 0.0, 1.0, 0.0)) and math.isnan(lib.kvfuse_threshold_for_rate(100.0, 0.0, 1.0, 100.0))
    # golden normal tail values
    for ln in open(os.path.join(ROOT, "tests", "golden", "normal_tail.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        z, tail = (float(x) for x in ln.split())
        assert lib.kvfuse_exceedance_rate(1.0, 0.0, 1.0, z) == pytest.approx(tail, rel=1e-13)
        assert th.exceedance_rate(1.0, 0.0, 1.0, z) == pytest.approx(tail, rel=1e-13)
    # corollary
    lib.kvfuse_predict_compression.argtypes = [ctypes.POINTER(f64), ctypes.c_int32, f64, ctypes.POINTER(f64), ctypes.POINTER(f64)]
    rates = [3.0, 0.25, 17.5, 0.0]
    arr, p0, cr = (f64 * 4)(*rates), (f64 * 4)(), f64(0.0)
    assert lib.kvfuse_predict_compression(arr, 4, 128.0, ctypes.byref(cr), p0) == 0
    want_cr, want_p0 = th.predicted_compression(rates, 128.0)
    assert cr.value == pytest.approx(want_cr, rel=1e-15) and list(p0) == pytest.approx(list(want_p0), rel=1e-15)
    for args in ((0.9, 2.0, 1.5, 0.1, 0.5, 0.99), (0.9, 1.1, 1.5, 0.1, 0.5, 0.99), (0.98, 9.0, 1.5, 0.5, 0.5, 0.99), (0.6, 1.0, 3.0, 0.5, 0.5, 0.99)):
        assert lib.kvfuse_threshold_feedback(*args) == pytest.approx(th.feedback_step(*args), rel=1e-15)
