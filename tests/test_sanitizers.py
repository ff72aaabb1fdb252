"""The oracle (plain C) and the host side of the HIP library under the address and undefined-behaviour sanitizers.
CPU only: sanitizers run on host code, never on the GPU.  The oracle build is driven by oracle/sanitize_driver.c on
a small seeded problem whose results must equal the ordinary build's; the library's host code (tree construction,
workspace layout, request ordering, closed forms, argument checks) is driven by csrc/host_check.cpp."""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2601_03067_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-4000:]}"
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, r.stdout[-4000:]
    return r.stdout


@pytest.mark.parametrize("rule", ["argmax", "first_row"])
def test_oracle_under_address_and_ub_sanitizers(oracle, rule):
    rec = wl.mixed(n_req=7, min_tokens=20, max_tokens=500, chunk_tokens=128, layers=1, kv_heads=1, pool=30, t=8, d=32)
    mat = wl.materialise(rec, "cpu", phys_perm=True)
    K, V, bt = wl.to_numpy_pool(mat["K"][0]), wl.to_numpy_pool(mat["V"][0]), mat["bt"][0].numpy().astype(np.int32)
    want = oracle.fuse_group(K, V, bt, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr, rule=rule)
    assert want.stats[1] > 0
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "ora_san")
        _run(["gcc", "-O1", "-g", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
              "-fno-sanitize-recover=undefined", "-static-libasan", "-o", exe, os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-lm"])
        P, r = K.shape
        with open(os.path.join(tmp, "in.bin"), "wb") as f:
            np.array([K.dtype.itemsize, r, P, len(bt), len(rec.leaf_start), len(rec.unit_leaf_ptr) - 1, rec.group_size,
                      {"argmax": 0, "first_row": 1}[rule]], np.int32).tofile(f)
            np.array([rec.thr, 1e-3], np.float64).tofile(f)
            for a in (K, V, bt, np.asarray(rec.leaf_start, np.int32), np.asarray(rec.leaf_count, np.int32),
                      np.asarray(rec.unit_leaf_ptr, np.int32)):
                np.ascontiguousarray(a).tofile(f)
        _run([exe, os.path.join(tmp, "in.bin"), os.path.join(tmp, "out.bin")])
        with open(os.path.join(tmp, "out.bin"), "rb") as f:
            got_bt = np.fromfile(f, np.int32, len(bt))
            got_rc = np.fromfile(f, np.int32, P)
            got_k = np.fromfile(f, K.dtype, P * r).reshape(P, r)
            got_v = np.fromfile(f, K.dtype, P * r).reshape(P, r)
            got_sk = np.fromfile(f, np.float64, len(bt))
            got_sv = np.fromfile(f, np.float64, len(bt))
            got_stats = np.fromfile(f, np.float64, 8)
    assert np.array_equal(got_bt, want.bt) and np.array_equal(got_rc, want.refcount)
    assert np.array_equal(got_k, want.kpool) and np.array_equal(got_v, want.vpool)
    assert np.array_equal(got_sk, want.scale_k) and np.array_equal(got_sv, want.scale_v)
    assert np.array_equal(got_stats, want.stats)


def test_library_host_code_under_address_and_ub_sanitizers():
    from paper_2601_03067_amd import build as kbuild
    hipcc = kbuild._hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    tmp = tempfile.mkdtemp(prefix="kvfuse_san_")
    try:
        def one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            _run([hipcc, *kbuild.FLAGS, "-O1", "-g", *san, "-c", src, "-o", obj])
            return obj
        srcs = [os.path.join(kbuild.CSRC, s) for s in kbuild.SOURCES]
        with ThreadPoolExecutor(max_workers=8) as ex:
            objs = list(ex.map(one, srcs))
        chk = os.path.join(tmp, "host_check.o")
        _run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-c",
              os.path.join(kbuild.CSRC, "host_check.cpp"), "-o", chk])
        exe = os.path.join(tmp, "host_check")
        _run([hipcc, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, chk, *objs])
        out = _run([exe])
        assert "host check passed" in out, out
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
