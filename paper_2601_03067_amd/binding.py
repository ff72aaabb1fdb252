"""ctypes binding of libkvfuse.so: the same entry points as include/kvfuse.h, argument marshalling only.

Every step of the hot path runs inside the HIP library.  PyTorch is used by callers for device memory and
streams; this module only turns tensors into pointers.  There is no fallback: if the library has not been
built (``python -m paper_2601_03067_amd.build``) importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvfuse.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_03067_amd.build` (needs hipcc)")
lib = C.CDLL(LIB_PATH)

OK, EINVAL, ESHAPE, EOVERFLOW, ENOMEM, EHIP = range(6)
F32, BF16 = 0, 1

EXPORTS = [
    "kvfuse_create", "kvfuse_destroy", "kvfuse_last_error", "kvfuse_workspace_bytes", "kvfuse_plan_create",
    "kvfuse_plan_destroy", "kvfuse_plan_heights", "kvfuse_plan_view", "kvfuse_block_norms", "kvfuse_leaf_sets",
    "kvfuse_similarity", "kvfuse_assign", "kvfuse_merge", "kvfuse_rewrite_block_table", "kvfuse_fuse_tree",
    "kvfuse_decode_workspace_bytes", "kvfuse_paged_decode_attn", "kvfuse_paged_decode_attn_static",
    "kvfuse_paged_decode_attn_all_heads",
]

_vp, _i32, _i64, _f32, _f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_double


class Pool(C.Structure):
    _fields_ = [("k", _vp), ("v", _vp), ("dtype", _i32), ("G", _i32), ("P", _i32), ("t", _i32), ("d", _i32),
                ("norm_k", _vp), ("norm_v", _vp), ("inv_norm_k", _vp)]


class Table(C.Structure):
    _fields_ = [("n", _i32), ("bt", _vp), ("scale_k", _vp), ("scale_v", _vp), ("orig_norm_k", _vp),
                ("orig_norm_v", _vp), ("refcount", _vp), ("remap", _vp)]


class TreeSpec(C.Structure):
    _fields_ = [("n_leaves", _i32), ("leaf_start", _vp), ("leaf_count", _vp), ("n_units", _i32),
                ("unit_leaf_ptr", _vp), ("group_size", _i32)]


class Stats(C.Structure):
    _fields_ = [("logical_blocks", _i64), ("physical_blocks", _i64), ("fused", _i64), ("near_threshold", _i64),
                ("refined", _i64), ("cand_overflow", _i64), ("compression_ratio", _f64), ("sim_flops", _f64),
                ("ms_norms", _f32), ("ms_similarity", _f32), ("ms_assign", _f32), ("ms_merge", _f32),
                ("ms_rewrite", _f32), ("ms_total", _f32), ("n_heights", _i32), ("merge_targets", _i32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class HeightView(C.Structure):
    _fields_ = [("n_nodes", _i32), ("total_l_cap", _i32), ("total_r_cap", _i32), ("cand_cap", _i32), ("total_s", _i64),
                ("l_off", _vp), ("r_off", _vp), ("l_slot", _vp), ("r_slot", _vp), ("out_slot", _vp), ("l_cap", _vp),
                ("r_cap", _vp), ("l_base", _vp), ("r_base", _vp), ("s_base", _vp), ("set_ids", _vp), ("set_cnt", _vp),
                ("assign", _vp), ("best_packed", _vp), ("cand_cnt", _vp), ("n_slots", _i32),
                ("r_stride", _i32), ("l_stride", _i32), ("reserved", _i32)]


lib.kvfuse_last_error.restype = C.c_char_p
lib.kvfuse_last_error.argtypes = [_vp]
lib.kvfuse_create.argtypes = [C.POINTER(_vp), C.c_int, _vp]
lib.kvfuse_destroy.argtypes = [_vp]
lib.kvfuse_workspace_bytes.argtypes = [_i32, _i32, C.POINTER(TreeSpec), _i32, C.POINTER(C.c_size_t)]
lib.kvfuse_plan_create.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), C.POINTER(TreeSpec), _i32, _vp, C.c_size_t,
                                   C.POINTER(_vp)]
lib.kvfuse_plan_destroy.argtypes = [_vp]
lib.kvfuse_plan_heights.argtypes = [_vp, C.POINTER(_i32)]
lib.kvfuse_plan_view.argtypes = [_vp, _i32, C.POINTER(HeightView)]
lib.kvfuse_block_norms.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table)]
lib.kvfuse_leaf_sets.argtypes = [_vp, _vp]
lib.kvfuse_similarity.argtypes = [_vp, _vp, _i32, _f64, _f64, _vp]
lib.kvfuse_assign.argtypes = [_vp, _vp, _i32, _f64, _f64]
lib.kvfuse_merge.argtypes = [_vp, _vp, _i32]
lib.kvfuse_rewrite_block_table.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _vp, _vp, _vp]
lib.kvfuse_fuse_tree.argtypes = [_vp, _vp, _f64, _f64, _vp, _vp, _vp, C.POINTER(Stats), _i32]
lib.kvfuse_decode_workspace_bytes.argtypes = [_i32, _i32, _i32, _i32, _i32, _i32, C.POINTER(C.c_size_t)]
lib.kvfuse_paged_decode_attn.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _i32, _i32, _i32, _vp, _vp, _vp, _i32,
                                         _i32, _i32, _f32, _vp, C.c_size_t, _vp]
lib.kvfuse_paged_decode_attn_all_heads.argtypes = lib.kvfuse_paged_decode_attn.argtypes
lib.kvfuse_paged_decode_attn_static.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _i32, _i32, _i32, _vp, _vp, _vp, _i32,
                                                _i32, _i32, _f32, _vp]
DECODE_STATIC_SCRATCH_BYTES = 8 << 20



class DecodePlanInfo(C.Structure):
    _fields_ = [("device_bytes", C.c_int64), ("clusters", C.c_int64), ("shared_instances", C.c_int64),
                ("logical_blocks", C.c_int64), ("cluster_block_reads", C.c_int64), ("residual_block_reads", C.c_int64),
                ("items_cluster", C.c_int64), ("items_residual", C.c_int64)]


lib.kvfuse_shared_decode_plan_build.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _i32, _i32, _i32, _vp, _vp, _i32, _i32,
                                                _i32, C.POINTER(_vp), C.POINTER(DecodePlanInfo)]
lib.kvfuse_shared_decode_plan_upload.argtypes = [_vp, _vp, _vp, C.c_size_t]
lib.kvfuse_shared_decode_plan_destroy.argtypes = [_vp]
lib.kvfuse_paged_decode_attn_shared.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _vp, _vp, C.c_float, _vp]


class PrefillPlanInfo(C.Structure):
    _fields_ = [("device_bytes", C.c_int64), ("logical_blocks_before_chunk", C.c_int64),
                ("stored_blocks_before_chunk", C.c_int64)]


lib.kvfuse_prefill_plan_build.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32,
                                          _i32, C.POINTER(_vp), C.POINTER(PrefillPlanInfo)]
lib.kvfuse_prefill_plan_upload.argtypes = [_vp, _vp, _vp, C.c_size_t]
lib.kvfuse_prefill_plan_destroy.argtypes = [_vp]
lib.kvfuse_prefill_attn.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _vp, _vp, C.c_float, _vp]
lib.kvfuse_pair_cosines.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _vp, _i32, _vp]
lib.kvfuse_cosine_moments.argtypes = [_vp, _vp, _i32, _i32, _vp]
lib.kvfuse_exceedance_rate.argtypes = [_f64, _f64, _f64, _f64]
lib.kvfuse_exceedance_rate.restype = _f64
lib.kvfuse_threshold_for_rate.argtypes = [_f64, _f64, _f64, _f64]
lib.kvfuse_threshold_for_rate.restype = _f64
lib.kvfuse_predict_compression.argtypes = [C.POINTER(_f64), _i32, _f64, C.POINTER(_f64), C.POINTER(_f64)]
lib.kvfuse_threshold_feedback.argtypes = [_f64] * 6
lib.kvfuse_threshold_feedback.restype = _f64
lib.kvfuse_plan_set_group_mask.argtypes = [_vp, _vp, _vp]
lib.kvfuse_plan_set_assign_rule.argtypes = [_vp, _vp, _i32]
lib.kvfuse_plan_group_counters.argtypes = [_vp, _vp, _vp, _i32]
lib.kvfuse_plan_set_screen_prefix.argtypes = [_vp, _vp, _i32, _vp]
lib.kvfuse_plan_set_screen_fp8.argtypes = [_vp, _vp, _vp, C.c_size_t, _vp, C.c_size_t, C.c_int32]
lib.kvfuse_tree_spec_shortest_first.argtypes = [C.POINTER(TreeSpec), _vp, _vp, _vp, _vp]
lib.kvfuse_replicate_rescaled.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table), _vp]
lib.kvfuse_drop_rescale.argtypes = [_vp, C.POINTER(Pool), C.POINTER(Table)]
RULE_ARGMAX, RULE_FIRST_ROW = 0, 1


class KvfuseError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"kvfuse error {code}: {text}")
        self.code = code


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dtype_code(dt):
    if dt == torch.bfloat16:
        return BF16
    if dt == torch.float32:
        return F32
    raise KvfuseError(ESHAPE, f"unsupported pool dtype {dt}")


class Context:
    """kvfuse_create / kvfuse_destroy on the current torch stream of ``device``."""

    def __init__(self, device="cuda:0", stream=None):
        dev = torch.device(device)
        self.device = dev
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        self.h = _vp()
        rc = lib.kvfuse_create(C.byref(self.h), dev.index or 0, C.c_void_p(self.stream.cuda_stream))
        if rc:
            raise KvfuseError(rc, "kvfuse_create failed")

    def check(self, rc):
        if rc:
            raise KvfuseError(rc, lib.kvfuse_last_error(self.h).decode())

    def close(self):
        if self.h:
            lib.kvfuse_destroy(self.h)
            self.h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Cache:
    """Device buffers of one paged KV cache plus the descriptor structs that point at them (allocation only)."""

    def __init__(self, K: torch.Tensor, V: torch.Tensor, bt: torch.Tensor, t: int, d: int):
        assert K.is_contiguous() and V.is_contiguous() and bt.is_contiguous() and K.shape == V.shape
        G, P, r = K.shape
        assert r == t * d and bt.shape[0] == G and bt.dtype == torch.int32
        dev = K.device
        n = bt.shape[1]
        self.K, self.V, self.bt, self.t, self.d, self.G, self.P, self.n = K, V, bt, t, d, G, P, n
        self.norm_k = torch.empty(G, P, device=dev, dtype=torch.float64)
        self.norm_v = torch.empty(G, P, device=dev, dtype=torch.float64)
        self.inv_norm_k = torch.empty(G, P, device=dev, dtype=torch.float32)
        self.scale_k = torch.empty(G, n, device=dev, dtype=torch.float32)
        self.scale_v = torch.empty(G, n, device=dev, dtype=torch.float32)
        self.orig_norm_k = torch.empty(G, n, device=dev, dtype=torch.float64)
        self.orig_norm_v = torch.empty(G, n, device=dev, dtype=torch.float64)
        self.refcount = torch.empty(G, P, device=dev, dtype=torch.int32)
        self.remap = torch.empty(G, P, device=dev, dtype=torch.int32)
        self.free_list = torch.empty(G, P, device=dev, dtype=torch.int32)
        self.n_free = torch.empty(G, device=dev, dtype=torch.int32)
        self.n_phys = torch.empty(G, device=dev, dtype=torch.int32)
        self.pool = Pool(_ptr(K), _ptr(V), _dtype_code(K.dtype), G, P, t, d, _ptr(self.norm_k), _ptr(self.norm_v),
                         _ptr(self.inv_norm_k))
        self.table = Table(n, _ptr(bt), _ptr(self.scale_k), _ptr(self.scale_v), _ptr(self.orig_norm_k),
                           _ptr(self.orig_norm_v), _ptr(self.refcount), _ptr(self.remap))

    def identity_scales(self):
        """Table state of an unfused cache (for decode attention without a fusion pass)."""
        self.scale_k.fill_(1.0)
        self.scale_v.fill_(1.0)


def tree_spec(leaf_start, leaf_count, unit_leaf_ptr, group_size=0):
    ls = np.ascontiguousarray(leaf_start, np.int32)
    lc = np.ascontiguousarray(leaf_count, np.int32)
    up = np.ascontiguousarray(unit_leaf_ptr, np.int32)
    spec = TreeSpec(len(ls), ls.ctypes.data, lc.ctypes.data, len(up) - 1, up.ctypes.data, int(group_size))
    spec._keep = (ls, lc, up)   # host arrays must outlive the struct
    return spec


def workspace_bytes(G, n, spec, cand_cap=64):
    out = C.c_size_t(0)
    rc = lib.kvfuse_workspace_bytes(G, n, C.byref(spec), cand_cap, C.byref(out))
    if rc:
        raise KvfuseError(rc, "kvfuse_workspace_bytes failed")
    return out.value


class Plan:
    """kvfuse_plan_create over a caller-allocated (torch) workspace."""

    def __init__(self, ctx: Context, cache: Cache, spec: TreeSpec, cand_cap: int = 64):
        self.ctx, self.cache, self.spec, self.cand_cap = ctx, cache, spec, cand_cap
        nbytes = workspace_bytes(cache.G, cache.n, spec, cand_cap)
        self.workspace = torch.empty(nbytes + 256, device=cache.K.device, dtype=torch.uint8)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.h = _vp()
        ctx.check(lib.kvfuse_plan_create(ctx.h, C.byref(cache.pool), C.byref(cache.table), C.byref(spec), cand_cap,
                                         C.c_void_p(base), nbytes, C.byref(self.h)))

    @property
    def n_heights(self):
        out = _i32(0)
        self.ctx.check(lib.kvfuse_plan_heights(self.h, C.byref(out)))
        return out.value

    def view(self, height):
        v = HeightView()
        self.ctx.check(lib.kvfuse_plan_view(self.h, height, C.byref(v)))
        return v

    def close(self):
        if self.h:
            lib.kvfuse_plan_destroy(self.h)
            self.h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def block_norms(ctx, cache):
    ctx.check(lib.kvfuse_block_norms(ctx.h, C.byref(cache.pool), C.byref(cache.table)))


def leaf_sets(ctx, plan):
    ctx.check(lib.kvfuse_leaf_sets(ctx.h, plan.h))


def similarity(ctx, plan, height, thr, band=1e-3, dense_s=None):
    ctx.check(lib.kvfuse_similarity(ctx.h, plan.h, height, thr, band, _ptr(dense_s)))


def assign(ctx, plan, height, thr, band=1e-3):
    ctx.check(lib.kvfuse_assign(ctx.h, plan.h, height, thr, band))


def merge(ctx, plan, height):
    ctx.check(lib.kvfuse_merge(ctx.h, plan.h, height))


def rewrite_block_table(ctx, cache, want_lists=True):
    ctx.check(lib.kvfuse_rewrite_block_table(ctx.h, C.byref(cache.pool), C.byref(cache.table),
                                             _ptr(cache.free_list) if want_lists else None,
                                             _ptr(cache.n_free) if want_lists else None,
                                             _ptr(cache.n_phys) if want_lists else None))


def fuse_tree(ctx, plan, thr, band=1e-3, want_stats=True, want_timing=False):
    cache = plan.cache
    st = Stats()
    ctx.check(lib.kvfuse_fuse_tree(ctx.h, plan.h, thr, band, _ptr(cache.free_list), _ptr(cache.n_free), _ptr(cache.n_phys),
                                   C.byref(st) if want_stats else None, 1 if want_timing else 0))
    return st if want_stats else None


def decode_workspace_bytes(n_layers, B, Hq, kv_heads, d, max_blocks):
    out = C.c_size_t(0)
    rc = lib.kvfuse_decode_workspace_bytes(n_layers, B, Hq, kv_heads, d, max_blocks, C.byref(out))
    if rc:
        raise KvfuseError(rc, "kvfuse_decode_workspace_bytes failed")
    return out.value


def paged_decode_attn(ctx, cache, kv_heads, q, req_start, ctx_len, max_blocks, layer_begin=0, sm_scale=None,
                      workspace=None, out=None):
    """q [n_layers][B][Hq][d] (pool dtype) -> out [n_layers][B][Hq][d] float32."""
    n_layers, B, Hq, d = q.shape
    assert q.is_contiguous() and q.dtype == cache.K.dtype and d == cache.d
    if sm_scale is None:
        sm_scale = 1.0 / float(d) ** 0.5
    if out is None:
        out = torch.empty(n_layers, B, Hq, d, device=q.device, dtype=torch.float32)
    nbytes = decode_workspace_bytes(n_layers, B, Hq, kv_heads, d, max_blocks)
    if workspace is None or workspace.numel() < nbytes:
        workspace = torch.empty(nbytes, device=q.device, dtype=torch.uint8)
    ctx.check(lib.kvfuse_paged_decode_attn(ctx.h, C.byref(cache.pool), C.byref(cache.table), kv_heads, layer_begin, n_layers,
                                           _ptr(q), _ptr(req_start), _ptr(ctx_len), B, Hq, max_blocks, sm_scale,
                                           _ptr(workspace), workspace.numel(), _ptr(out)))
    return out


def paged_decode_attn_all_heads(ctx, cache, kv_heads, q, req_start, ctx_len, max_blocks, layer_begin=0, sm_scale=None,
                                workspace=None, out=None):
    """Decode through a cache of all-head blocks: cache.K/V are [layers][P][t * kv_heads * head size], cache.d =
    kv_heads * head size, one table per layer.  q [n_layers][B][Hq][head size] -> out float32, same shape."""
    n_layers, B, Hq, hd = q.shape
    assert q.is_contiguous() and q.dtype == cache.K.dtype and hd * kv_heads == cache.d
    if sm_scale is None:
        sm_scale = 1.0 / float(hd) ** 0.5
    if out is None:
        out = torch.empty(n_layers, B, Hq, hd, device=q.device, dtype=torch.float32)
    nbytes = decode_workspace_bytes(n_layers, B, Hq, kv_heads, hd, max_blocks)
    if workspace is None or workspace.numel() < nbytes:
        workspace = torch.empty(nbytes, device=q.device, dtype=torch.uint8)
    ctx.check(lib.kvfuse_paged_decode_attn_all_heads(ctx.h, C.byref(cache.pool), C.byref(cache.table), kv_heads, layer_begin,
                                                     n_layers, _ptr(q), _ptr(req_start), _ptr(ctx_len), B, Hq, max_blocks,
                                                     sm_scale, _ptr(workspace), workspace.numel(), _ptr(out)))
    return out


def paged_decode_attn_static(ctx, cache, kv_heads, q, req_start, ctx_len, max_blocks, out, layer_begin=0, sm_scale=None):
    """kvfuse_paged_decode_attn_static: the caller passes inputs and the output; nothing is allocated on the way."""
    n_layers, B, Hq, d = q.shape
    assert q.is_contiguous() and q.dtype == cache.K.dtype and d == cache.d
    assert out.is_contiguous() and out.dtype == torch.float32 and tuple(out.shape) == (n_layers, B, Hq, d)
    if sm_scale is None:
        sm_scale = 1.0 / float(d) ** 0.5
    ctx.check(lib.kvfuse_paged_decode_attn_static(ctx.h, C.byref(cache.pool), C.byref(cache.table), kv_heads, layer_begin,
                                                  n_layers, _ptr(q), _ptr(req_start), _ptr(ctx_len), B, Hq, max_blocks,
                                                  sm_scale, _ptr(out)))
    return out


class PrefillPlan:
    """Plan for kvfuse_prefill_attn: queries = tokens [q_begin, q_end) of the chunk starting at chunk_begin."""

    def __init__(self, ctx, cache, kv_heads, Hq, req_start, chunk_begin, q_begin, q_end, layer_begin=0, n_layers=None,
                 reuse=True):
        self.ctx = ctx
        self.h = _vp()
        if n_layers is None:
            n_layers = cache.pool.G // kv_heads - layer_begin
        self.n_layers, self.Hq, self.nq = n_layers, Hq, q_end - q_begin
        self.info = PrefillPlanInfo()
        ctx.check(lib.kvfuse_prefill_plan_build(ctx.h, C.byref(cache.pool), C.byref(cache.table), kv_heads, layer_begin, n_layers,
                                                int(req_start), int(chunk_begin), int(q_begin), int(q_end), Hq, 1 if reuse else 0,
                                                C.byref(self.h), C.byref(self.info)))
        self.workspace = torch.empty(int(self.info.device_bytes), device=cache.K.device, dtype=torch.uint8)
        ctx.check(lib.kvfuse_prefill_plan_upload(ctx.h, self.h, _ptr(self.workspace), self.workspace.numel()))

    def close(self):
        if getattr(self, "h", None):
            lib.kvfuse_prefill_plan_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def prefill_attn(ctx, cache, plan, q, sm_scale=None, out=None):
    """q [n_layers][Nq][Hq][d] bfloat16 -> out float32 of the same shape (causal attention through the table)."""
    n_layers, nq, Hq, d = q.shape
    assert q.is_contiguous() and q.dtype == cache.K.dtype and d == cache.d and (n_layers, nq, Hq) == (plan.n_layers, plan.nq, plan.Hq)
    if sm_scale is None:
        sm_scale = 1.0 / float(d) ** 0.5
    if out is None:
        out = torch.empty(n_layers, nq, Hq, d, device=q.device, dtype=torch.float32)
    ctx.check(lib.kvfuse_prefill_attn(ctx.h, C.byref(cache.pool), C.byref(cache.table), plan.h, _ptr(q), sm_scale, _ptr(out)))
    return out


def pair_cosines(ctx, cache, pairs, out=None):
    """pairs: int32 tensor [n_pairs][2] of logical indices (device) -> float64 tensor [G][n_pairs] of key cosines."""
    assert pairs.dtype == torch.int32 and pairs.is_contiguous() and pairs.dim() == 2 and pairs.shape[1] == 2
    n_pairs = pairs.shape[0]
    if out is None:
        out = torch.empty(cache.pool.G, n_pairs, device=pairs.device, dtype=torch.float64)
    ctx.check(lib.kvfuse_pair_cosines(ctx.h, C.byref(cache.pool), C.byref(cache.table), _ptr(pairs), n_pairs, _ptr(out)))
    return out


def cosine_moments(ctx, cos):
    """float64 [G][n_pairs] -> float64 [G][2] (mean, population variance)."""
    assert cos.dtype == torch.float64 and cos.is_contiguous() and cos.dim() == 2
    out = torch.empty(cos.shape[0], 2, device=cos.device, dtype=torch.float64)
    ctx.check(lib.kvfuse_cosine_moments(ctx.h, _ptr(cos), cos.shape[0], cos.shape[1], _ptr(out)))
    return out


def exceedance_rate(n, mu, sigma, u):
    return lib.kvfuse_exceedance_rate(n, mu, sigma, u)


def threshold_for_rate(n, mu, sigma, rate):
    return lib.kvfuse_threshold_for_rate(n, mu, sigma, rate)


def predict_compression(rates, blocks_per_layer):
    """-> (compression ratio, [probability of no fusion per layer])."""
    L = len(rates)
    arr = (_f64 * L)(*[float(r) for r in rates])
    p0 = (_f64 * L)()
    cr = _f64(0.0)
    rc = lib.kvfuse_predict_compression(arr, L, float(blocks_per_layer), C.byref(cr), p0)
    if rc:
        raise KvfuseError(rc, "kvfuse_predict_compression: bad arguments")
    return cr.value, list(p0)


def threshold_feedback(thr, observed_cr, target_cr, gain, lo, hi):
    return lib.kvfuse_threshold_feedback(thr, observed_cr, target_cr, gain, lo, hi)


def set_group_mask(ctx, plan, enable):
    """enable: uint8 tensor [G] on the device (kept alive by the plan object), or None for all groups."""
    if enable is not None:
        assert enable.dtype == torch.uint8 and enable.is_contiguous() and enable.numel() == plan.cache.pool.G
    plan.group_mask = enable
    ctx.check(lib.kvfuse_plan_set_group_mask(ctx.h, plan.h, _ptr(enable) if enable is not None else None))


def set_screen_prefix(ctx, plan, prefix_elements):
    """kvfuse_plan_set_screen_prefix; allocates the [G][P] tail-share array the call needs and keeps it with the plan."""
    if prefix_elements:
        plan.tail_share = torch.empty(plan.cache.G, plan.cache.P, device=plan.cache.K.device, dtype=torch.float32)
        ctx.check(lib.kvfuse_plan_set_screen_prefix(ctx.h, plan.h, int(prefix_elements), _ptr(plan.tail_share)))
    else:
        ctx.check(lib.kvfuse_plan_set_screen_prefix(ctx.h, plan.h, 0, None))
        plan.tail_share = None


def set_screen_fp8(ctx, plan, on=True, centre=False):
    """kvfuse_plan_set_screen_fp8; allocates the one-byte copy of the key pool and its side array and keeps them with the
    plan: plan.k8 [G][P][r] bytes, and views plan.k8_err / k8_scale / k8_alpha [G][P] and plan.k8_dir [G][r] of the side
    array."""
    if on:
        c = plan.cache
        r = c.t * c.d
        k8 = torch.empty(c.G, c.P, r, device=c.K.device, dtype=torch.uint8)
        side = torch.zeros(3 * c.G * c.P + c.G * r, device=c.K.device, dtype=torch.float32)
        ctx.check(lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, _ptr(k8), k8.numel(), _ptr(side), side.numel(), 1 if centre else 0))
        gp = c.G * c.P
        plan.k8, plan.k8_side = k8, side
        plan.k8_err = side[:gp].view(c.G, c.P)
        plan.k8_scale = side[gp:2 * gp].view(c.G, c.P)
        plan.k8_alpha = side[2 * gp:3 * gp].view(c.G, c.P)
        plan.k8_dir = side[3 * gp:].view(c.G, r)
    else:
        ctx.check(lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, None, 0, None, 0, 0))
        plan.k8 = plan.k8_side = plan.k8_err = plan.k8_scale = plan.k8_alpha = plan.k8_dir = None


def group_counters(ctx, plan):
    """kvfuse_plan_group_counters -> numpy [G][4]: fused, near-threshold, refined in fp64, candidate overflow, per group."""
    out = np.zeros((plan.cache.G, 4), np.int32)
    ctx.check(lib.kvfuse_plan_group_counters(ctx.h, plan.h, out.ctypes.data, plan.cache.G))
    return out


def set_assign_rule(ctx, plan, rule):
    ctx.check(lib.kvfuse_plan_set_assign_rule(ctx.h, plan.h, int(rule)))


def tree_spec_shortest_first(spec: TreeSpec):
    """-> (reordered TreeSpec, order): units (leaves, when there is one unit) in ascending number of blocks."""
    ls = np.zeros(max(spec.n_leaves, 1), np.int32)
    lc = np.zeros(max(spec.n_leaves, 1), np.int32)
    up = np.zeros(spec.n_units + 1, np.int32)
    order = np.zeros(max(spec.n_leaves if spec.n_units == 1 else spec.n_units, 1), np.int32)
    rc = lib.kvfuse_tree_spec_shortest_first(C.byref(spec), ls.ctypes.data, lc.ctypes.data, up.ctypes.data,
                                             order.ctypes.data)
    if rc:
        raise KvfuseError(rc, "kvfuse_tree_spec_shortest_first failed")
    n_order = spec.n_leaves if spec.n_units == 1 else spec.n_units
    return tree_spec(ls[:spec.n_leaves], lc[:spec.n_leaves], up, spec.group_size), order[:n_order].copy()


def replicate_rescaled(ctx, cache, orig_bt):
    """orig_bt: int32 tensor [G][n] on the device, the table before fusion."""
    assert orig_bt.dtype == torch.int32 and orig_bt.is_contiguous() and orig_bt.shape == cache.bt.shape
    ctx.check(lib.kvfuse_replicate_rescaled(ctx.h, C.byref(cache.pool), C.byref(cache.table), _ptr(orig_bt)))


def drop_rescale(ctx, cache):
    ctx.check(lib.kvfuse_drop_rescale(ctx.h, C.byref(cache.pool), C.byref(cache.table)))


class SharedDecodePlan:
    """Decode plan for kvfuse_paged_decode_attn_shared, built from the cache's current table (rebuild after a fusion)."""

    def __init__(self, ctx, cache, kv_heads, req_start, ctx_len, Hq, layer_begin=0, n_layers=None, min_cluster_blocks=4):
        import numpy as np
        self.ctx = ctx
        self.h = _vp()
        rs = np.ascontiguousarray(np.asarray(req_start.cpu() if hasattr(req_start, "cpu") else req_start, dtype=np.int32))
        cl = np.ascontiguousarray(np.asarray(ctx_len.cpu() if hasattr(ctx_len, "cpu") else ctx_len, dtype=np.int32))
        if n_layers is None:
            n_layers = cache.pool.G // kv_heads - layer_begin
        self.n_layers, self.B, self.Hq, self.kv_heads = n_layers, len(rs), Hq, kv_heads
        self.info = DecodePlanInfo()
        ctx.check(lib.kvfuse_shared_decode_plan_build(ctx.h, C.byref(cache.pool), C.byref(cache.table), kv_heads, layer_begin,
                                                      n_layers, rs.ctypes.data_as(_vp), cl.ctypes.data_as(_vp), len(rs), Hq,
                                                      min_cluster_blocks, C.byref(self.h), C.byref(self.info)))
        self.workspace = torch.empty(int(self.info.device_bytes), device=cache.K.device, dtype=torch.uint8)
        ctx.check(lib.kvfuse_shared_decode_plan_upload(ctx.h, self.h, _ptr(self.workspace), self.workspace.numel()))

    def close(self):
        if getattr(self, "h", None):
            lib.kvfuse_shared_decode_plan_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the module globals may already be gone
            pass


def paged_decode_attn_shared(ctx, cache, plan, q, sm_scale=None, out=None):
    """q [n_layers][B][Hq][d] (pool dtype) -> out [n_layers][B][Hq][d] float32, through a SharedDecodePlan."""
    n_layers, B, Hq, d = q.shape
    assert q.is_contiguous() and q.dtype == cache.K.dtype and d == cache.d
    assert (n_layers, B, Hq) == (plan.n_layers, plan.B, plan.Hq)
    if sm_scale is None:
        sm_scale = 1.0 / float(d) ** 0.5
    if out is None:
        out = torch.empty(n_layers, B, Hq, d, device=q.device, dtype=torch.float32)
    ctx.check(lib.kvfuse_paged_decode_attn_shared(ctx.h, C.byref(cache.pool), C.byref(cache.table), plan.h, _ptr(q), sm_scale,
                                                  _ptr(out)))
    return out


def unpack_best(packed):
    """Column maxima as stored by the similarity step -> (cosine float32 array, row int64 array; row -1 = none)."""
    packed = np.asarray(packed, np.uint64)
    ordered = (packed >> np.uint64(32)).astype(np.uint32)
    bits = np.where(ordered & np.uint32(0x80000000), ordered & np.uint32(0x7FFFFFFF), ~ordered)
    val = bits.astype(np.uint32).view(np.float32)
    row = (np.uint64(0xFFFFFFFF) - (packed & np.uint64(0xFFFFFFFF))).astype(np.int64)
    none = packed == 0
    return np.where(none, np.float32(-np.inf), val), np.where(none, -1, row)


_hip = None


def device_array(ptr, count, dtype, device):
    """Copy ``count`` elements of a device array given by raw pointer into a host numpy array (tests, tools)."""
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [_vp, _vp, C.c_size_t, C.c_int]
    torch.cuda.synchronize(device)
    out = np.empty(count, dtype=dtype)
    if count:
        rc = _hip.hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)   # hipMemcpyDeviceToHost
        if rc != 0:
            raise KvfuseError(EHIP, f"hipMemcpy failed: {rc}")
    return out
