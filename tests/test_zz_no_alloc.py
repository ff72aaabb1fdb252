"""GPU test of kvfuse_paged_decode_attn_static, the decode entry point that allocates nothing: its split-KV partial
states live in a static device array of the library.  It must give what kvfuse_paged_decode_attn gives with a caller
workspace (same kernels, same launch shape: bit-equal), on two calls in a row that share the array, the second one
smaller, and must refuse a call whose partial states do not fit."""
import numpy as np
import pytest
import torch

from paper_2601_03067_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(kb, rec):
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    assert stats.fused > 0
    q = wl.queries(rec, DEV)
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=DEV)
    cl = torch.tensor(rec.ctx_len, dtype=torch.int32, device=DEV)
    mb = int(((rec.ctx_len + rec.t - 1) // rec.t).max())
    return ctx, cache, q, rs, cl, mb


def test_static_scratch_decode_equals_workspace_decode(oracle):
    kb = gu.load_binding()
    # long contexts and few (layer, request, KV head) tuples: the launch splits every context, so the partial states
    # (the scratch) are really used; the second call is smaller and must not see what the first one left behind
    big = wl.cff_long(tokens=16 * 700, chunk_tokens=16 * 100, layers=1, kv_heads=2)
    small = wl.llama8b_bff(n_req=3, tokens=16 * 41, layers=1, kv_heads=2, prefix_tokens=64, near_pool=16)
    for name, rec in (("first call, 700 blocks of context", big), ("second call, smaller", small)):
        print("static-scratch decode:", name, flush=True)
        ctx, cache, q, rs, cl, mb = _inputs(kb, rec)
        need = kb.decode_workspace_bytes(rec.layers, rec.B, rec.q_heads, rec.kv_heads, rec.d, mb)
        assert 256 < need <= kb.DECODE_STATIC_SCRATCH_BYTES, need      # split-KV launch, and it fits
        ref = kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, mb)
        out = torch.full_like(ref, float("nan"))
        kb.paged_decode_attn_static(ctx, cache, rec.kv_heads, q, rs, cl, mb, out)
        torch.cuda.synchronize()
        assert torch.equal(out, ref), float((out - ref).abs().max())
        # and against the oracle, to the decode bar
        gs = list(range(rec.kv_heads))
        att = oracle.paged_decode_attention(
            q[0].float().cpu().numpy().astype(np.float64), [wl.to_numpy_pool(cache.K[g]) for g in gs],
            [wl.to_numpy_pool(cache.V[g]) for g in gs], [cache.bt[g].cpu().numpy() for g in gs],
            [cache.scale_k[g].cpu().numpy().astype(np.float64) for g in gs],
            [cache.scale_v[g].cpu().numpy().astype(np.float64) for g in gs], rec.req_start, rec.ctx_len, rec.t, rec.d)
        err = float(np.abs(out[0].cpu().numpy() - att).max())
        print("  max abs err against the oracle", err, flush=True)
        assert err <= 5e-3


def test_static_scratch_decode_rejects_what_does_not_fit():
    kb = gu.load_binding()
    rec = wl.llama8b_bff(n_req=3, tokens=16 * 41, layers=1, kv_heads=2, prefix_tokens=64, near_pool=16)
    ctx, cache, _, _, _, _ = _inputs(kb, rec)
    # 1024 (request, KV head) tuples of 16 query heads each, split in two: 17 MB of partial states.  The host check
    # refuses before anything is launched, so the request arrays are never read.
    B, Hq, mb = 512, 16 * rec.kv_heads, 64
    assert kb.decode_workspace_bytes(1, B, Hq, rec.kv_heads, rec.d, mb) > kb.DECODE_STATIC_SCRATCH_BYTES
    q = torch.zeros(1, B, Hq, rec.d, device=DEV, dtype=cache.K.dtype)
    rs = torch.zeros(B, device=DEV, dtype=torch.int32)
    out = torch.empty(1, B, Hq, rec.d, device=DEV, dtype=torch.float32)
    with pytest.raises(kb.KvfuseError) as ei:
        kb.paged_decode_attn_static(ctx, cache, rec.kv_heads, q, rs, rs, mb, out)
    assert ei.value.code == kb.ENOMEM and "static array holds" in str(ei.value)
