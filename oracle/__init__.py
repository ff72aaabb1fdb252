"""CPU oracle for the Fast Fusion hot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
(``paper_2601_03067_amd``) and never imports it.

Two parts:

* ``kvfuse_oracle.c`` (plain C, fp64, one accumulator): block norms, the
  similarity / threshold / fusion / block-table steps of Algorithm 1 and the
  recursion itself, for one (layer, KV head) group at a time.  This module
  compiles it with gcc and wraps it with ctypes.  Groups are independent, so
  the wrapper may run several groups on host threads; nothing inside a group
  is parallel.
* ``paged_decode_attention`` (numpy, fp64): softmax attention of one query per
  request over the logical blocks of that request, each logical block being
  ``scale * stored(bt[x])`` (method section: one shared unit direction plus a
  norm per logical block; analysis section: logits q.k/sqrt(d)).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvfuse_oracle.c")
_LIB = os.path.join(_HERE, "libkvfuse_oracle.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc.  No fast-math: fp64 order is the definition."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ora_test_round_bf16.restype = ctypes.c_double
        _lib.ora_test_round_bf16.argtypes = [ctypes.c_double]
        _lib.ora_fuse_group.restype = ctypes.c_int
    return _lib


def _ptr(a: np.ndarray, ty=ctypes.c_void_p):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ty)


def _elem_bytes(pool: np.ndarray) -> int:
    if pool.dtype == np.float32:
        return 4
    if pool.dtype == np.uint16:  # bfloat16 bit patterns
        return 2
    raise TypeError("pool must be float32 or uint16 (bfloat16 bits)")


def round_bf16(x: float) -> float:
    return _load().ora_test_round_bf16(float(x))


def pool_to_f64(pool: np.ndarray) -> np.ndarray:
    """Exact widening of a pool tensor (float32 or bfloat16 bits) to float64."""
    if pool.dtype == np.uint16:
        return (pool.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return pool.astype(np.float64)


# ----------------------------------------------------------------------
# single steps of one node (used by per-step tests)
# ----------------------------------------------------------------------

def block_norms(pool: np.ndarray) -> np.ndarray:
    """pool [P][r] -> norm [P] fp64 (method section: the norm of each block vector is stored)."""
    lib = _load()
    P, r = pool.shape
    out = np.zeros(P, np.float64)
    lib.ora_block_norms(_ptr(pool), _elem_bytes(pool), r, P, _ptr(out, _f64p))
    return out


def similarity(kpool: np.ndarray, norm_k: np.ndarray, L: np.ndarray, R: np.ndarray) -> np.ndarray:
    """Dense cosine matrix S[ml][mr] of one node (Algorithm 1, similarity line)."""
    lib = _load()
    L = np.ascontiguousarray(L, np.int32)
    R = np.ascontiguousarray(R, np.int32)
    S = np.zeros((len(L), len(R)), np.float64)
    lib.ora_similarity(_ptr(kpool), _elem_bytes(kpool), kpool.shape[1], _ptr(norm_k, _f64p),
                       _ptr(L, _i32p), len(L), _ptr(R, _i32p), len(R), _ptr(S, _f64p))
    return S


def assign(S: np.ndarray, thr: float):
    """Thresholded arg-max per right block -> (assign[mr], best[mr], second[mr])."""
    lib = _load()
    S = np.ascontiguousarray(S, np.float64)
    ml, mr = S.shape
    a = np.full(mr, -1, np.int32)
    best = np.zeros(mr, np.float64)
    second = np.zeros(mr, np.float64)
    lib.ora_assign(_ptr(S, _f64p), ml, mr, ctypes.c_double(thr), _ptr(a, _i32p), _ptr(best, _f64p),
                   _ptr(second, _f64p))
    return a, best, second


def assign_first_row(S: np.ndarray, thr: float):
    """Threshold line of Algorithm 1 in row order: the first row above thr takes the block -> assign[mr]."""
    lib = _load()
    S = np.ascontiguousarray(S, np.float64)
    ml, mr = S.shape
    a = np.full(mr, -1, np.int32)
    lib.ora_assign_first_row(_ptr(S, _f64p), ml, mr, ctypes.c_double(thr), _ptr(a, _i32p))
    return a


def merge(pool: np.ndarray, norm: np.ndarray, L, R, assign_) -> None:
    """Fusion lines of Algorithm 1 for one pool tensor, in place (pool rows and norm of targets)."""
    lib = _load()
    L = np.ascontiguousarray(L, np.int32)
    R = np.ascontiguousarray(R, np.int32)
    a = np.ascontiguousarray(assign_, np.int32)
    lib.ora_merge(_ptr(pool), _elem_bytes(pool), pool.shape[1], _ptr(norm, _f64p), _ptr(L, _i32p), len(L),
                  _ptr(R, _i32p), len(R), _ptr(a, _i32p))


def rewrite(bt, L, R, assign_, orig_norm_k, orig_norm_v, norm_k, norm_v, scale_k, scale_v, refcount):
    """Evict / update block-table step, in place.  Returns the evicted ids in eviction order."""
    lib = _load()
    L = np.ascontiguousarray(L, np.int32)
    R = np.ascontiguousarray(R, np.int32)
    a = np.ascontiguousarray(assign_, np.int32)
    free_list = np.zeros(len(refcount), np.int32)
    n_free = ctypes.c_int32(0)
    lib.ora_rewrite(_ptr(bt, _i32p), len(bt), _ptr(L, _i32p), len(L), _ptr(R, _i32p), len(R), _ptr(a, _i32p),
                    _ptr(orig_norm_k, _f64p), _ptr(orig_norm_v, _f64p), _ptr(norm_k, _f64p), _ptr(norm_v, _f64p),
                    _ptr(scale_k, _f64p), _ptr(scale_v, _f64p), _ptr(refcount, _i32p), _ptr(free_list, _i32p),
                    ctypes.byref(n_free))
    return free_list[: n_free.value].copy()


# ----------------------------------------------------------------------
# the whole recursion for one group / many groups
# ----------------------------------------------------------------------

class GroupResult:
    """Outputs of Fast Fusion for one group (all numpy, fp64 where floating)."""

    __slots__ = ("kpool", "vpool", "bt", "orig_norm_k", "orig_norm_v", "norm_k", "norm_v", "scale_k",
                 "scale_v", "refcount", "free_list", "stats", "trace")

    @property
    def n_physical(self) -> int:
        return int(self.stats[6])

    @property
    def compression_ratio(self) -> float:
        return float(self.stats[7])


def fuse_group(kpool: np.ndarray, vpool: np.ndarray, bt: np.ndarray, leaf_start, leaf_count, unit_leaf_ptr,
               thr: float, group_size: int = 0, band: float = 1e-3, want_trace: bool = False,
               rule: str = "argmax") -> GroupResult:
    """Run Algorithm 1 on one group.  Inputs are copied; the result holds the fused pool and table.
    rule: "argmax" (one target per right block, the most similar row) or "first_row" (the row loop taken
    literally: the first row above the threshold takes the block)."""
    lib = _load()
    eb = _elem_bytes(kpool)
    assert kpool.shape == vpool.shape and kpool.dtype == vpool.dtype
    P, r = kpool.shape
    res = GroupResult()
    res.kpool = np.array(kpool, copy=True, order="C")
    res.vpool = np.array(vpool, copy=True, order="C")
    res.bt = np.array(bt, dtype=np.int32, copy=True, order="C")
    n = len(res.bt)
    ls = np.ascontiguousarray(leaf_start, np.int32)
    lc = np.ascontiguousarray(leaf_count, np.int32)
    ul = np.ascontiguousarray(unit_leaf_ptr, np.int32)
    res.orig_norm_k = np.zeros(n, np.float64)
    res.orig_norm_v = np.zeros(n, np.float64)
    res.norm_k = np.zeros(P, np.float64)
    res.norm_v = np.zeros(P, np.float64)
    res.scale_k = np.zeros(n, np.float64)
    res.scale_v = np.zeros(n, np.float64)
    res.refcount = np.zeros(P, np.int32)
    free_list = np.zeros(P, np.int32)
    n_free = ctypes.c_int32(0)
    res.stats = np.zeros(8, np.float64)
    trace_cap = 2 * n * 64 if want_trace else 0
    trace = np.zeros(max(trace_cap, 1), np.int32)
    trace_len = ctypes.c_int64(0)
    rc = lib.ora_fuse_group(
        eb, r, P, n, _ptr(res.kpool), _ptr(res.vpool), _ptr(res.bt, _i32p),
        _ptr(ls, _i32p), _ptr(lc, _i32p), len(ls), _ptr(ul, _i32p), len(ul) - 1, int(group_size),
        ctypes.c_double(thr), ctypes.c_double(band),
        _ptr(res.orig_norm_k, _f64p), _ptr(res.orig_norm_v, _f64p), _ptr(res.norm_k, _f64p),
        _ptr(res.norm_v, _f64p), _ptr(res.scale_k, _f64p), _ptr(res.scale_v, _f64p),
        _ptr(res.refcount, _i32p), _ptr(free_list, _i32p), ctypes.byref(n_free), _ptr(res.stats, _f64p),
        _ptr(trace, _i32p) if want_trace else None, ctypes.c_int64(trace_cap), ctypes.byref(trace_len),
        {"argmax": 0, "first_row": 1}[rule])
    if rc != 0:
        raise ValueError(f"ora_fuse_group failed with code {rc}")
    res.free_list = free_list[: n_free.value].copy()
    res.trace = trace[: trace_len.value].reshape(-1, 2).copy() if want_trace else None
    return res


def set_column_threads(n: int) -> None:
    """Host threads that share out the (independent) columns of one tree node; 1 = none.  For groups too large to
    walk on one core in reasonable time.  Changes the run time only: every cosine stays one left-to-right fp64 sum.
    Process-wide; do not combine with ``fuse_groups(threads > 1)``."""
    _load().ora_set_column_threads(int(n))


def fuse_groups(kpools, vpools, bts, leaf_start, leaf_count, unit_leaf_ptr, thr, group_size=0, band=1e-3,
                threads: int = 1, rule: str = "argmax"):
    """Independent groups on ``threads`` host threads (ctypes drops the GIL inside the C call)."""
    def one(g):
        return fuse_group(kpools[g], vpools[g], bts[g], leaf_start, leaf_count, unit_leaf_ptr, thr,
                          group_size, band, rule=rule)
    G = len(kpools)
    if threads <= 1:
        return [one(g) for g in range(G)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(one, range(G)))


# ----------------------------------------------------------------------
# variants: order of the requests, the two evaluation modes
# ----------------------------------------------------------------------

def shortest_first(leaf_start, leaf_count, unit_leaf_ptr):
    """Remark after Algorithm 1: requests with fewer blocks go to the left of the tree.  Units in ascending
    number of blocks, ties in their given order, each unit keeping its leaves; with one unit its leaves are
    ordered instead.  -> (leaf_start, leaf_count, unit_leaf_ptr, order)."""
    ls, lc, up = (np.asarray(a, np.int64) for a in (leaf_start, leaf_count, unit_leaf_ptr))
    n_units = len(up) - 1
    if n_units == 1:
        order = sorted(range(len(ls)), key=lambda l: (lc[l], l))
        return ls[order].astype(np.int32), lc[order].astype(np.int32), up.astype(np.int32), np.asarray(order, np.int32)
    size = [int(lc[up[u]:up[u + 1]].sum()) for u in range(n_units)]
    order = sorted(range(n_units), key=lambda u: (size[u], u))
    out_s, out_c, out_p = [], [], [0]
    for u in order:
        out_s += list(ls[up[u]:up[u + 1]])
        out_c += list(lc[up[u]:up[u + 1]])
        out_p.append(len(out_s))
    return (np.asarray(out_s, np.int32), np.asarray(out_c, np.int32), np.asarray(out_p, np.int32),
            np.asarray(order, np.int32))


def _round_to_pool(x: np.ndarray, like: np.ndarray) -> np.ndarray:
    """fp64 -> the pool's storage type, nearest even, one rounding."""
    lib = _load()
    flat = np.ascontiguousarray(x, np.float64).ravel()
    out = np.empty(flat.shape, like.dtype)
    lib.ora_store_array(_ptr(out), _elem_bytes(like), _ptr(flat, _f64p), ctypes.c_size_t(flat.size))
    return out.reshape(x.shape)


def replicate_rescaled(pool: np.ndarray, bt0: np.ndarray, bt: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """First evaluation mode of the results section for one pool tensor of one group: every logical block x gets
    the block it had before fusion, bt0[x], filled with scale[x] * stored(bt[x]) in the pool's type; nothing is
    freed.  The scale is the binary32 number the table holds.  Returns the new pool [P][r]; blocks that no entry
    of bt0 names are unchanged."""
    src = pool_to_f64(pool)
    out = np.array(pool, copy=True)
    for x in range(len(bt0)):
        s = float(np.float32(scale[x]))
        out[bt0[x]] = _round_to_pool(s * src[bt[x]], pool)
    return out


# ----------------------------------------------------------------------
# decode attention through a (possibly fused) block table
# ----------------------------------------------------------------------

def paged_decode_attention(q, kpool, vpool, bt, scale_k, scale_v, req_start, ctx_len, t, d, sm_scale=None):
    """Textbook softmax attention, one query per request, fp64.

    q         [B][Hq][d]     queries of ONE layer
    kpool     [H][P][t*d]    pool of that layer, one slab per KV head (float32 or bfloat16 bits)
    bt        [H][n]         per-group block table; request b owns logical entries
                             req_start[b] .. req_start[b] + ceil(ctx_len[b] / t)
    scale_*   [H][n]         per-logical-block rescale
    ctx_len   [B]            tokens of context; the last block may be partial
    Query head h reads KV head h // (Hq // H).
    Logits z = sm_scale * scale_k[x] * <q, K[bt[x]][tok]>, out = sum softmax(z) * scale_v[x] * V[bt[x]][tok].
    """
    q = np.asarray(q, np.float64)
    B, Hq, dd = q.shape
    assert dd == d
    H = len(kpool)
    rep = Hq // H
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    out = np.zeros((B, Hq, d), np.float64)
    for b in range(B):
        T = int(ctx_len[b])
        if T == 0:
            continue
        nb = (T + t - 1) // t
        for h in range(Hq):
            g = h // rep
            xs = np.arange(req_start[b], req_start[b] + nb)
            phys = np.asarray(bt[g])[xs]
            kb = pool_to_f64(np.asarray(kpool[g])[phys]).reshape(nb, t, d) * np.asarray(scale_k[g], np.float64)[xs, None, None]
            vb = pool_to_f64(np.asarray(vpool[g])[phys]).reshape(nb, t, d) * np.asarray(scale_v[g], np.float64)[xs, None, None]
            kt = kb.reshape(nb * t, d)[:T]
            vt = vb.reshape(nb * t, d)[:T]
            z = sm_scale * (kt @ q[b, h])
            z = z - z.max()
            p = np.exp(z)
            p /= p.sum()
            out[b, h] = p @ vt
    return out


def causal_prefill_attention(q, q_pos, kpool, vpool, bt, scale_k, scale_v, req_start, t, d, sm_scale=None):
    """Textbook causal softmax attention of a run of query tokens of ONE request over its paged context, fp64
    (motivation section: chunked prefill over a cache whose table points several logical blocks at one stored
    block; the query at position pos sees the tokens 0 .. pos of its own request).

    q         [Nq][Hq][d]    queries of ONE layer, query i sits at absolute token position q_pos[i]
    kpool     [H][P][t*d]    pool of that layer, one slab per KV head (float32 or bfloat16 bits)
    bt        [H][n]         per-group block table; the request owns logical entries req_start, req_start + 1, ...
    scale_*   [H][n]         per-logical-block rescale
    Query head h reads KV head h // (Hq // H).  Token tau lives in logical block x = req_start + tau // t:
    z_tau = sm_scale * scale_k[x] * <q, K[bt[x]][tau % t]>, out = sum_{tau <= pos} softmax(z)_tau * scale_v[x] * V[bt[x]][tau % t].
    """
    q = np.asarray(q, np.float64)
    Nq, Hq, dd = q.shape
    assert dd == d
    H = len(kpool)
    rep = Hq // H
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    q_pos = np.asarray(q_pos, np.int64)
    T = int(q_pos.max()) + 1
    nb = (T + t - 1) // t
    out = np.zeros((Nq, Hq, d), np.float64)
    for g in range(H):
        xs = np.arange(req_start, req_start + nb)
        phys = np.asarray(bt[g])[xs]
        kt = (pool_to_f64(np.asarray(kpool[g])[phys]).reshape(nb, t, d) * np.asarray(scale_k[g], np.float64)[xs, None, None]).reshape(nb * t, d)
        vt = (pool_to_f64(np.asarray(vpool[g])[phys]).reshape(nb, t, d) * np.asarray(scale_v[g], np.float64)[xs, None, None]).reshape(nb * t, d)
        for i in range(Nq):
            L = int(q_pos[i]) + 1
            for h in range(g * rep, (g + 1) * rep):
                z = sm_scale * (kt[:L] @ q[i, h])
                z = z - z.max()
                p = np.exp(z)
                p /= p.sum()
                out[i, h] = p @ vt[:L]
    return out
