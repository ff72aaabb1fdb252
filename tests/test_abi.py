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
PROBE_HEADER = os.path.join(ROOT, "include", "kvfuse_probe.h")
LIB = os.path.join(ROOT, "paper_2601_03067_amd", "libkvfuse.so")
PROBE_LIB = os.path.join(ROOT, "paper_2601_03067_amd", "libkvfuse_probe.so")


def _declared(header=HEADER):
    text = open(header).read()
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


def test_probe_library_is_separate_and_exports_its_header(lib):
    """The machine probes are bench tooling: their own header and shared library, nothing of them in the product."""
    names = _declared(PROBE_HEADER)
    assert len(names) == 6 and all(n.startswith("kvfuse_probe_") for n in names)
    plib = ctypes.CDLL(PROBE_LIB)
    assert not [n for n in names if not hasattr(plib, n)]
    assert not [n for n in names if hasattr(lib, n)]
    assert not [n for n in _declared() if "probe" in n]
    assert plib.kvfuse_probe_copy(None, None, None, 0, 1, None) == 1      # bad arguments are an error code, no GPU needed


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


class _Spec(ctypes.Structure):
    _fields_ = [("n_leaves", ctypes.c_int32), ("leaf_start", ctypes.c_void_p), ("leaf_count", ctypes.c_void_p),
                ("n_units", ctypes.c_int32), ("unit_leaf_ptr", ctypes.c_void_p), ("group_size", ctypes.c_int32)]


def _shortest_first(lib, ls, lc, up):
    ls, lc, up = (np.ascontiguousarray(a, np.int32) for a in (ls, lc, up))
    spec = _Spec(len(ls), ls.ctypes.data, lc.ctypes.data, len(up) - 1, up.ctypes.data, 0)
    o_ls, o_lc, o_up = np.zeros_like(ls), np.zeros_like(lc), np.zeros_like(up)
    order = np.zeros(len(ls) if len(up) == 2 else len(up) - 1, np.int32)
    lib.kvfuse_tree_spec_shortest_first.argtypes = [ctypes.POINTER(_Spec)] + [ctypes.c_void_p] * 4
    rc = lib.kvfuse_tree_spec_shortest_first(ctypes.byref(spec), o_ls.ctypes.data, o_lc.ctypes.data, o_up.ctypes.data,
                                             order.ctypes.data)
    return rc, o_ls, o_lc, o_up, order


def test_shortest_first_order_matches_the_oracle(lib):
    """Host-only entry point (remark on the order of requests): compared with the oracle's ordering on random specs,
    with and without several leaves per unit, and on the one-unit case."""
    import oracle
    rng = np.random.default_rng(41)
    for case in range(60):
        n_units = 1 if case % 5 == 0 else int(rng.integers(2, 12))
        per_unit = rng.integers(0 if n_units > 1 else 1, 4, size=n_units)
        lc = rng.integers(0, 6, size=int(per_unit.sum())).astype(np.int32)      # ties and empty leaves on purpose
        ls = np.concatenate([[0], np.cumsum(lc)[:-1]]).astype(np.int32) if len(lc) else np.zeros(0, np.int32)
        up = np.concatenate([[0], np.cumsum(per_unit)]).astype(np.int32)
        rc, o_ls, o_lc, o_up, order = _shortest_first(lib, ls, lc, up)
        assert rc == 0
        w_ls, w_lc, w_up, w_order = oracle.shortest_first(ls, lc, up)
        assert o_ls.tolist() == w_ls.tolist() and o_lc.tolist() == w_lc.tolist() and o_up.tolist() == w_up.tolist()
        assert order.tolist() == w_order.tolist()
        # a permutation of the same leaves, sizes non-decreasing
        assert sorted(zip(o_ls.tolist(), o_lc.tolist())) == sorted(zip(ls.tolist(), lc.tolist()))
        if n_units > 1:
            sizes = [int(o_lc[o_up[u]:o_up[u + 1]].sum()) for u in range(n_units)]
            assert sizes == sorted(sizes)
    assert lib.kvfuse_tree_spec_shortest_first(None, None, None, None, None) != 0


def test_variant_entry_points_reject_null_arguments(lib):
    assert lib.kvfuse_plan_set_assign_rule(None, None, 1) != 0
    assert lib.kvfuse_replicate_rescaled(None, None, None, None) != 0
    assert lib.kvfuse_drop_rescale(None, None, None) != 0


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++) on its own."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "include/kvfuse.h"\nint main(void) { kvfuse_stats s; (void)s; return KVFUSE_OK; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", ROOT, str(src)])
    if shutil.which("g++") is not None:
        subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", ROOT, str(src)])
