"""GPU test: the fusion pass and a decode step recorded in a HIP graph.

A serving loop replays one graph per step instead of launching some forty kernels.  kvfuse_fuse_tree (without
statistics, which need a host read) and kvfuse_paged_decode_attn launch kernels on the context's stream and nothing
else: no allocation, no host synchronisation, no memset node.  So they can be recorded.  The graph here restores the
pool and the table from saved copies, fuses and decodes; it is replayed several times with eager work between the
replays that overwrites everything the graph reads or writes, and every replay must leave exactly what the eager
calls left: tables, pools, scales and attention outputs bit-equal (the eager path is compared with the oracle in
test_gpu_parity.py, and once more here)."""
import numpy as np
import pytest
import torch

from paper_2601_03067_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _state(cache, out):
    return [t.clone() for t in (cache.K, cache.V, cache.bt, cache.scale_k, cache.scale_v, cache.refcount, cache.n_phys, out)]


@pytest.mark.parametrize("screen", ["full_product", "prefix_256", "fp8_copies", "fp8_copies_centred"])
def test_fusion_and_decode_replayed_from_a_graph(oracle, screen):
    kb = gu.load_binding()
    rec = wl.llama8b_bff(n_req=6, tokens=16 * 150, layers=1, kv_heads=3, prefix_tokens=192, near_pool=24, t=16, d=64)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    host = gu.host_copy(mat)
    K0, V0, bt0 = mat["K"].clone(), mat["V"].clone(), mat["bt"].clone()
    side = torch.cuda.Stream(DEV)
    q = wl.queries(rec, DEV)
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=DEV)
    cl = torch.tensor(rec.ctx_len, dtype=torch.int32, device=DEV)
    mb = int(((rec.ctx_len + rec.t - 1) // rec.t).max())
    out = torch.empty(rec.layers, rec.B, rec.q_heads, rec.d, device=DEV, dtype=torch.float32)
    ws = torch.empty(max(kb.decode_workspace_bytes(rec.layers, rec.B, rec.q_heads, rec.kv_heads, rec.d, mb), 256),
                     device=DEV, dtype=torch.uint8)
    torch.cuda.synchronize()

    with torch.cuda.stream(side):
        ctx = kb.Context(DEV, stream=side)
        cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
        plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr), 16)
        if screen == "prefix_256":
            kb.set_screen_prefix(ctx, plan, 256)
        elif screen.startswith("fp8_copies"):
            kb.set_screen_fp8(ctx, plan, centre=screen.endswith("centred"))

        def step():
            cache.K.copy_(K0)
            cache.V.copy_(V0)
            cache.bt.copy_(bt0)
            kb.fuse_tree(ctx, plan, rec.thr, want_stats=False)
            kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, mb, workspace=ws, out=out)

        print("graph test: eager step", flush=True)
        step()          # eager: the reference, and every one-time set-up of the library happens here
        side.synchronize()
        want = _state(cache, out)

        # the eager result is what the oracle gives
        res = gu.oracle_fuse(oracle, rec, host)
        assert gu.check_ambiguity(res, "graph_eager") == list(range(rec.G))
        for g in range(rec.G):
            gu.compare_group(res[g], cache, g, False, "graph_eager")
        assert sum(int(r.stats[1]) for r in res) > 50

        print("graph test: capture", flush=True)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for replay in range(3):
            # eager work between the replays: everything the graph writes is overwritten first
            cache.K.fill_(0.25)
            cache.V.fill_(-3.0)
            cache.bt.fill_(0)
            cache.scale_k.fill_(7.0)
            cache.scale_v.fill_(7.0)
            out.fill_(float("nan"))
            side.synchronize()
            print("graph test: replay", replay, flush=True)
            graph.replay()
            side.synchronize()
            got = _state(cache, out)
            for name, a, b in zip(("K", "V", "bt", "scale_k", "scale_v", "refcount", "n_phys", "attention"), got, want):
                assert torch.equal(a, b), (replay, name)
    assert np.isfinite(want[-1].cpu().numpy()).all()
