"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: block tables, assignments, reference counts, free lists and fused pool bytes bit-exact; norms 1e-13
relative (fp64 sums in a different order); scales 2e-7 relative (fp32 storage); screened cosines within the
screen's stated error band; attention within 2e-2 max-abs (checked much tighter where fp32 allows).
"""
import ctypes as C
import math

import numpy as np
import pytest
import torch

from paper_2601_03067_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def kb():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return gu.load_binding()


def _small_bf16(n_req=6, tokens=1200, layers=1, kv_heads=3, t=8, d=32, near_pool=24, prefix_tokens=96, seed=wl.MASTER_SEED):
    """Llama-shaped recipe shrunk so that the oracle takes seconds: r = 256, 150 blocks per request (ragged vs the
    128-wide tiles of the similarity kernel)."""
    return wl.llama8b_bff(n_req=n_req, tokens=tokens, layers=layers, kv_heads=kv_heads, prefix_tokens=prefix_tokens,
                          near_pool=near_pool, t=t, d=d, seed=seed)


# ------------------------------------------------------------------------------------------ a1 norms

@pytest.mark.parametrize("which", ["tiny_f32", "small_bf16"])
def test_block_norms_match_oracle(kb, oracle, which):
    rec = wl.tiny_bff() if which == "tiny_f32" else _small_bf16()
    _say("norms", which, "G", rec.G, "n", rec.n, "r", rec.r)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    kb.block_norms(ctx, cache)
    torch.cuda.synchronize()
    for g in range(rec.G):
        nk = oracle.block_norms(wl.to_numpy_pool(mat["K"][g]))
        nv = oracle.block_norms(wl.to_numpy_pool(mat["V"][g]))
        np.testing.assert_allclose(cache.norm_k[g].cpu().numpy(), nk, rtol=1e-14)
        np.testing.assert_allclose(cache.norm_v[g].cpu().numpy(), nv, rtol=1e-14)
        np.testing.assert_allclose(cache.inv_norm_k[g].cpu().numpy(), 1.0 / nk, rtol=1e-6)
        bt = mat["bt"][g].cpu().numpy()
        np.testing.assert_allclose(cache.orig_norm_k[g].cpu().numpy(), nk[bt], rtol=1e-14)
        assert (cache.scale_k[g] == 1).all() and (cache.refcount[g] == 1).all() and (cache.remap[g] == -1).all()


# ------------------------------------------------------------------------------------------ a2..a5 one node at a time

def _two_leaf_case(kind):
    """One tree node: left leaf and right leaf with planted duplicates, ragged against the 128 x 128 tiles
    (or, for the *_big kinds, against the 256 x 256 tiles with several row tiles and column panels)."""
    rng = np.random.default_rng({"f32": 5, "bf16": 6, "f32_big": 7, "bf16_big": 8, "bf16_common": 9}[kind])
    ml, mr = {"bf16": (150, 201), "f32": (70, 45), "bf16_big": (700, 530), "f32_big": (300, 290), "bf16_common": (150, 201)}[kind]
    r = 256 if kind.startswith("bf16") else 96
    n = ml + mr
    protos = rng.standard_normal((40, r))
    x = rng.standard_normal((n, r))
    pick = rng.integers(0, 40, n)
    dup = rng.random(n) < 0.5
    x[dup] = protos[pick[dup]] + 0.05 * rng.standard_normal((int(dup.sum()), r))
    x[ml + 3] = x[7]                      # exact duplicate across the node
    x[ml + 4] = x[7]                      # two right blocks for one target
    x[9] = x[8]                           # identical left rows: lowest row must win
    x[ml + 5] = x[8] + 1e-4 * rng.standard_normal(r)
    if kind == "bf16_common":             # every block shares a strong component: unrelated blocks at cosine 0.8
        x += 2.0 * rng.standard_normal(r)[None]
    x[11] = 0.0                           # zero blocks on both sides
    x[ml + 6] = 0.0
    y = rng.standard_normal((n, r))
    dt = torch.bfloat16 if kind.startswith("bf16") else torch.float32
    K = torch.tensor(x, dtype=torch.float32).to(dt)[None].contiguous()
    V = torch.tensor(y, dtype=torch.float32).to(dt)[None].contiguous()
    perm = rng.permutation(n)
    Kp, Vp = torch.empty_like(K), torch.empty_like(V)
    Kp[0][perm] = K[0]
    Vp[0][perm] = V[0]
    bt = torch.tensor(perm, dtype=torch.int32)[None].contiguous()
    t, d = (8, 32) if kind.startswith("bf16") else (4, 24)
    return Kp, Vp, bt, ml, mr, t, d


@pytest.mark.parametrize("kind", ["f32", "bf16", "f32_big", "bf16_big"])
@pytest.mark.parametrize("cand_cap", [16, 1])
def test_single_node_steps_match_oracle(kb, oracle, kind, cand_cap):
    _say("single node", kind, "cand_cap", cand_cap)
    K, V, bt, ml, mr, t, d = _two_leaf_case(kind)
    thr, band = 0.9, 1e-3
    Kh, Vh, bth = wl.to_numpy_pool(K[0]), wl.to_numpy_pool(V[0]), bt[0].numpy().copy()
    K, V, bt = K.to(DEV), V.to(DEV), bt.to(DEV)
    ctx = kb.Context(DEV)
    cache = kb.Cache(K, V, bt, t, d)
    spec = kb.tree_spec([0, ml], [ml, mr], [0, 1, 2])
    plan = kb.Plan(ctx, cache, spec, cand_cap)
    assert plan.n_heights == 1
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)
    view = plan.view(0)
    dense = torch.full((1, view.total_s), float("nan"), device=DEV)
    kb.similarity(ctx, plan, 0, thr, band, dense)
    torch.cuda.synchronize()

    # oracle, step by step
    nk, nv = oracle.block_norms(Kh), oracle.block_norms(Vh)
    L, R = bth[:ml], bth[ml:]
    S = oracle.similarity(Kh, nk, L, R)
    S_gpu = dense[0].cpu().numpy().reshape(ml, mr).astype(np.float64)
    err = np.abs(S_gpu - S).max()
    _say("  screen max |cos_gpu - cos_oracle| =", err)
    assert err <= Kh.shape[1] * 2.0 ** -22, "screen error exceeds the bound the fp64 re-check relies on"
    best, best_row = kb.unpack_best(kb.device_array(view.best_packed, mr, np.uint64, DEV))
    assert np.abs(best - S.max(0)).max() <= 1e-4
    clear = np.sort(S, 0)[-1] - np.sort(S, 0)[-2] > 1e-3          # columns whose maximum is unambiguous
    assert np.array_equal(best_row[clear], S.argmax(0)[clear])
    cnt = kb.device_array(view.cand_cnt, mr, np.int32, DEV)
    lo, hi = (S > thr - 2 * band + 1e-4).sum(0), (S > thr - 2 * band - 1e-4).sum(0)
    assert (cnt >= lo).all() and (cnt <= hi).all()
    assert cand_cap == 16 or (cnt > 1).any(), "the cand_cap = 1 case must exercise the overflow rescan"

    kb.assign(ctx, plan, 0, thr, band)
    torch.cuda.synchronize()
    a_or, best_or, second_or = oracle.assign(S, thr)
    a_gpu = kb.device_array(view.assign, mr, np.int32, DEV)
    assert (a_or >= 0).sum() >= 10
    assert np.array_equal(a_gpu, a_or), f"assignments differ at {np.nonzero(a_gpu != a_or)[0]}"
    # survivors = cat(left, non-fused right)
    slots = kb.device_array(view.set_cnt, view.n_slots, np.int32, DEV)
    out_slot = kb.device_array(view.out_slot, 1, np.int32, DEV)[0]
    want_set = np.concatenate([L, R[a_or < 0]])
    assert slots[out_slot] == len(want_set)
    assert np.array_equal(kb.device_array(view.set_ids, len(want_set), np.int32, DEV), want_set)

    kb.merge(ctx, plan, 0)
    kb.rewrite_block_table(ctx, cache)
    torch.cuda.synchronize()
    Ko, Vo = Kh.copy(), Vh.copy()
    nko, nvo = nk.copy(), nv.copy()
    oracle.merge(Ko, nko, L, R, a_or)
    oracle.merge(Vo, nvo, L, R, a_or)
    bto = bth.copy()
    sk, sv = np.ones(len(bto)), np.ones(len(bto))
    rc = np.ones(len(nk), np.int32)
    freed = oracle.rewrite(bto, L, R, a_or, nk[bth], nv[bth], nko, nvo, sk, sv, rc)
    Kg, Vg = wl.to_numpy_pool(cache.K[0]), wl.to_numpy_pool(cache.V[0])
    live = np.unique(bto)
    assert np.array_equal(Kg[live], Ko[live]) and np.array_equal(Vg[live], Vo[live]), "fused blocks differ from the oracle"
    assert np.array_equal(cache.bt[0].cpu().numpy(), bto)
    assert np.array_equal(cache.refcount[0].cpu().numpy(), rc)
    assert sorted(freed.tolist()) == cache.free_list[0, : int(cache.n_free[0])].cpu().numpy().tolist()
    np.testing.assert_allclose(cache.scale_k[0].cpu().numpy(), sk, rtol=2e-7)
    np.testing.assert_allclose(cache.scale_v[0].cpu().numpy(), sv, rtol=2e-7)
    np.testing.assert_allclose(cache.norm_k[0].cpu().numpy()[live], nko[live], rtol=1e-13)


# ------------------------------------------------------------------------------------------ whole tree

def _run_tree_case(kb, oracle, rec, name, cand_cap=16, thr=None, phys_perm=True, group_size=None, groups=None, band=1e-3,
                   rule="argmax", shortest_first=False, screen_prefix=0, screen_fp8=False):
    _say("tree case", name, "G", rec.G, "n", rec.n, "r", rec.r, "leaves", len(rec.leaf_start), "cand_cap", cand_cap,
         "rule", rule, "shortest_first", shortest_first)
    mat = wl.materialise(rec, DEV, groups=groups, phys_perm=phys_perm)
    host = gu.host_copy(mat)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, thr=thr, cand_cap=cand_cap, group_size=group_size, band=band, rule=rule,
                                          shortest_first=shortest_first, screen_prefix=screen_prefix, screen_fp8=screen_fp8)
    res = gu.oracle_fuse(oracle, rec, host, thr=thr, group_size=group_size, rule=rule, shortest_first=shortest_first)
    safe = gu.check_ambiguity(res, name)
    assert len(safe) == len(res)
    for g in safe:
        gu.compare_group(res[g], cache, g, rec.dtype == torch.float32, name)
    if len(safe) == len(res):
        assert stats.fused == sum(int(r.stats[1]) for r in res)
        assert stats.near_threshold == sum(int(r.stats[2]) for r in res)
        assert stats.physical_blocks == sum(r.n_physical for r in res)
        assert math.isclose(stats.compression_ratio, sum(len(r.bt) for r in res) / sum(r.n_physical for r in res))
    # the same counters group by group
    per_group = kb.group_counters(ctx, plan)
    assert per_group[:, 0].tolist() == [int(r.stats[1]) for r in res] and per_group[:, 1].tolist() == [int(r.stats[2]) for r in res]
    assert int(per_group[:, 2].sum()) == stats.refined and int(per_group[:, 3].sum()) == stats.cand_overflow
    _say("  fused", stats.fused, "refined", stats.refined, "overflow", stats.cand_overflow, "CR", round(stats.compression_ratio, 4))
    return cache, plan, stats, res, mat


def test_tree_tiny_config_all_groups(kb, oracle):
    """Config 1 as specified: fp32, 2 groups, 4 requests x 8 blocks, thr 0.95 -> 22 physical blocks per group."""
    rec = wl.tiny_bff()
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "tiny_bff")
    assert stats.physical_blocks == 2 * 22 and stats.fused == 20 and stats.near_threshold == 0
    assert stats.merge_targets == 20                      # ten disjoint pairs per group: one rebuilt block per fused one
    assert math.isclose(stats.compression_ratio, 32 / 22)


@pytest.mark.parametrize("screen_fp8", [False, True])
def test_tree_rescaling_blocks_by_powers_of_two_changes_only_the_scales(kb, screen_fp8):
    """The direction-plus-norm representation on the GPU path: every block times its own power of two (exact) gives the
    same table, the same fused representatives bit for bit, and scales that carry exactly that factor."""
    rec = _small_bf16(n_req=5, tokens=8 * 90, kv_heads=2)
    mat_a = wl.materialise(rec, DEV, phys_perm=True)
    mat_b = wl.materialise(rec, DEV, phys_perm=True)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(31)
    fk = (2.0 ** torch.randint(-6, 7, (rec.G, rec.n, 1), generator=gen).float()).to(DEV)
    fv = (2.0 ** torch.randint(-6, 7, (rec.G, rec.n, 1), generator=gen).float()).to(DEV)
    mat_b["K"] = (mat_b["K"].float() * fk).to(rec.dtype)
    mat_b["V"] = (mat_b["V"].float() * fv).to(rec.dtype)
    assert torch.equal((mat_b["K"].float() / fk).to(rec.dtype), mat_a["K"])
    bt0 = mat_a["bt"].clone().long()
    ca, pa, sa, _ = gu.gpu_fuse(rec, mat_a, screen_fp8=screen_fp8)
    cb, pb, sb, _ = gu.gpu_fuse(rec, mat_b, screen_fp8=screen_fp8)
    assert sa.fused == sb.fused > 50 and torch.equal(ca.bt, cb.bt) and torch.equal(ca.refcount, cb.refcount)
    for g in range(rec.G):
        fused = ca.refcount[g] > 1
        assert torch.equal(ca.K[g][fused], cb.K[g][fused]) and torch.equal(ca.V[g][fused], cb.V[g][fused])
        moved = fused[ca.bt[g].long()]
        fkx, fvx = fk[g, bt0[g], 0], fv[g, bt0[g], 0]            # factor of the block entry x had before fusion
        assert torch.equal(cb.scale_k[g][moved], ca.scale_k[g][moved] * fkx[moved])
        assert torch.equal(cb.scale_v[g][moved], ca.scale_v[g][moved] * fvx[moved])
        assert bool((cb.scale_k[g][~moved] == 1).all())


def test_tree_threshold_above_one_is_identity(kb, oracle):
    rec = wl.tiny_bff()
    mat = wl.materialise(rec, DEV)
    K0, V0 = mat["K"].clone(), mat["V"].clone()
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, thr=1.5)
    assert stats.fused == 0 and stats.compression_ratio == 1.0
    assert torch.equal(cache.K, K0) and torch.equal(cache.V, V0)
    assert torch.equal(cache.bt, torch.arange(rec.n, device=DEV, dtype=torch.int32).expand(rec.G, -1))
    assert (cache.scale_k == 1).all() and (cache.scale_v == 1).all() and (cache.refcount == 1).all()
    assert (cache.n_free == 0).all() and (cache.n_phys == rec.n).all()


@pytest.mark.parametrize("cand_cap", [16, 2])
def test_tree_small_bf16_bff(kb, oracle, cand_cap):
    """Six ragged-vs-tile requests of 150 blocks, shared prefix + near-duplicate pool, several tiles per node."""
    _run_tree_case(kb, oracle, _small_bf16(), "small_bf16_bff", cand_cap=cand_cap)


def test_tree_many_short_requests(kb, oracle):
    """600 requests of 3 blocks: 300 nodes at the lowest height, more than one workgroup's worth of nodes in the kernels
    that lay out the similarity work items of a height, 10 heights, and sets that stay far below their capacities."""
    rec = wl.llama8b_bff(n_req=600, tokens=8 * 3, layers=1, kv_heads=2, prefix_tokens=8, near_pool=40, near_frac=0.5, t=8, d=32,
                         dtype=torch.bfloat16, seed=77)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "bff_600_short_requests")
    assert plan.n_heights == 10 and stats.fused > 1000


def test_tree_seven_requests_non_power_of_two(kb, oracle):
    _run_tree_case(kb, oracle, _small_bf16(n_req=7, tokens=520, kv_heads=2), "bff_7_requests")


def test_tree_group_size(kb, oracle):
    rec = _small_bf16(n_req=8, tokens=400, kv_heads=2)
    _run_tree_case(kb, oracle, rec, "bff_group_size_3", group_size=3)


def test_tree_cff_chunks(kb, oracle):
    rec = wl.cff_long(tokens=8 * 600, chunk_tokens=8 * 75, layers=1, kv_heads=2, t=8, d=32)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "cff_small")
    assert stats.fused > 50


def test_tree_mixed_chunks_then_requests(kb, oracle):
    rec = wl.mixed(n_req=9, min_tokens=40, max_tokens=900, chunk_tokens=256, layers=1, kv_heads=2, pool=48, t=8, d=32)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "mixed_small")
    assert stats.fused > 50
    # partial tail blocks are in no leaf: they keep their own block and scale 1
    for b in range(rec.B):
        if rec.ctx_len[b] % rec.t:
            x = rec.req_start[b] + rec.req_blocks[b] - 1
            assert int(cache.refcount[0, cache.bt[0, x]]) == 1 and float(cache.scale_k[0, x]) == 1.0


def test_tree_zipf_many_near_ties(kb, oracle):
    """Config 4's structure shrunk: every block is a noisy copy of a Zipf-drawn base, so most right blocks have
    several near-tied left candidates and the fp64 re-check decides."""
    rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, thr=0.9)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "zipf_small", cand_cap=8)
    assert stats.refined > 20


def test_tree_zipf_threshold_in_the_thick_of_the_cosines(kb, oracle):
    """The same structure with the threshold at the cosine two noisy copies of one base have, 1 / (1 + sigma^2):
    most decisions lie within the screen's band of the threshold and are settled by the fp64 re-check."""
    sigma = 0.05
    rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, sigma=sigma,
                      thr=1.0 / (1.0 + sigma * sigma))
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "zipf_at_threshold", cand_cap=16)
    assert stats.refined > 100 and stats.near_threshold > 100


@pytest.mark.parametrize("rule", ["argmax", "first_row"])
@pytest.mark.parametrize("which", ["small_bf16_quarter", "small_bf16_half_cap2", "zipf_small_quarter", "zipf_at_threshold_half",
                                   "mixed_small_f32_quarter", "r4096_bf16_eighth", "tiny_too_short_a_prefix"])
def test_tree_prefix_screen_gives_the_same_tables(kb, oracle, which, rule):
    """The prefix screen (similarity over the first p elements of every key block + a Cauchy-Schwarz bound on the tails,
    every candidate evaluated in full in fp64) must give exactly the oracle's tables, pools and counters: with a prefix
    that rejects nearly everything (a quarter of random blocks), with few candidate slots (overflow -> column rescans),
    on near-tied Zipf copies, with the threshold in the thick of the cosines, on binary32 pools, on long blocks, under
    both readings of the threshold line, and with a prefix far too short for the data (every pair a candidate)."""
    kw = dict(rule=rule)
    if which == "small_bf16_quarter":
        rec, kw = _small_bf16(), dict(kw, screen_prefix=64)
    elif which == "small_bf16_half_cap2":
        rec, kw = _small_bf16(n_req=5, tokens=900), dict(kw, screen_prefix=128, cand_cap=2)
    elif which == "zipf_small_quarter":
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, thr=0.9)
        kw = dict(kw, screen_prefix=512, cand_cap=8)
    elif which == "zipf_at_threshold_half":
        sigma = 0.05
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, sigma=sigma,
                          thr=1.0 / (1.0 + sigma * sigma))
        kw = dict(kw, screen_prefix=1024)
    elif which == "mixed_small_f32_quarter":
        rec = wl.mixed(n_req=9, min_tokens=40, max_tokens=900, chunk_tokens=256, layers=1, kv_heads=2, pool=48, t=8, d=32,
                       dtype=torch.float32)
        kw = dict(kw, screen_prefix=64)
    elif which == "r4096_bf16_eighth":
        rec = wl.zipf_bff(n_req=6, tokens=32 * 150, layers=1, kv_heads=2, pool=400, t=32, d=128, thr=0.95)
        kw = dict(kw, screen_prefix=512, cand_cap=8)
    else:
        rec, kw = wl.tiny_bff(), dict(kw, screen_prefix=64, cand_cap=4)       # 64 of 1024 elements at thr 0.95: the bound rejects nothing
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "prefix_screen_" + which, **kw)
    assert stats.fused > 0
    if which == "tiny_too_short_a_prefix":
        assert stats.cand_overflow > 0


def test_prefix_screen_step_by_step_equals_the_tree_driver(kb, oracle):
    """The same tree walked through the single-step entry points (norms, leaf sets, then similarity / assignment / merge
    per height, rewrite) with the prefix screen on: the tail shares then come from kvfuse_leaf_sets and from the merge
    step, not from the driver's norm pass.  Must equal the oracle like the driver's result."""
    rec = _small_bf16(n_req=5, tokens=1000, kv_heads=2)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    host = gu.host_copy(mat)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr), 16)
    kb.set_screen_prefix(ctx, plan, 64)
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)
    for h in range(plan.n_heights):
        kb.similarity(ctx, plan, h, rec.thr)
        kb.assign(ctx, plan, h, rec.thr)
        kb.merge(ctx, plan, h)
    kb.rewrite_block_table(ctx, cache)
    torch.cuda.synchronize()
    res = gu.oracle_fuse(oracle, rec, host)
    assert gu.check_ambiguity(res, "prefix_step_by_step") == list(range(rec.G))
    for g in range(rec.G):
        gu.compare_group(res[g], cache, g, False, "prefix_step_by_step")
    assert sum(int(r.stats[1]) for r in res) > 50


# OCP e4m3 (4 exponent bits, bias 7, 3 mantissa bits, no infinities, 0x7F / 0xFF = NaN), written out from the format's
# definition: what the bytes of the fp8 screen's copy mean.
def _e4m3_table():
    out = np.zeros(256, np.float64)
    for b in range(256):
        e, m = (b >> 3) & 15, b & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = m / 8.0 * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        out[b] = -v if b & 0x80 else v
    return out


@pytest.mark.parametrize("centre", [False, True])
@pytest.mark.parametrize("kind", ["bf16", "bf16_big", "bf16_common"])
def test_fp8_screen_copy_and_bound(kb, oracle, kind, centre):
    """The fp8 screen's ingredients on one node.  With u the unit block, m the group's direction (zero when the copies
    are not centred), alpha = <m, u> and u_c = u - alpha m: the one-byte copy is the e4m3 rounding of u_c * 256 / |u_c|
    (checked against the format written out above: every byte decodes to within half a spacing of its element), the
    stored scale is |u_c| / 256, the stored error covers the copy's true Euclidean error plus what a non-unit m and the
    rounding of alpha cost (all recomputed here in fp64 from the bytes and the stored direction), and the kernel's value
    <q(a), q(b)> scale_a scale_b + alpha_a alpha_b stays within err_a + err_b + err_a err_b of the oracle's cosine for
    every pair -- the inequality the screen's candidate rule rests on."""
    K, V, bt, ml, mr, t, d = _two_leaf_case(kind)
    Kh, bth = wl.to_numpy_pool(K[0]), bt[0].numpy().copy()
    K, V, bt = K.to(DEV), V.to(DEV), bt.to(DEV)
    ctx = kb.Context(DEV)
    cache = kb.Cache(K, V, bt, t, d)
    plan = kb.Plan(ctx, cache, kb.tree_spec([0, ml], [ml, mr], [0, 1, 2]), 16)
    kb.set_screen_fp8(ctx, plan, centre=centre)
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)
    view = plan.view(0)
    dense = torch.full((1, view.total_s), float("nan"), device=DEV)
    kb.similarity(ctx, plan, 0, 0.9, 1e-3, dense)
    torch.cuda.synchronize()
    nk = oracle.block_norms(Kh)
    dec = _e4m3_table()[plan.k8[0].cpu().numpy()]                 # [P][r]
    assert np.isfinite(dec).all()
    live = nk > 0
    Kf = oracle.pool_to_f64(Kh)
    P, r = Kf.shape
    unit = np.zeros_like(Kf)
    unit[live] = Kf[live] / nk[live, None]
    m = plan.k8_dir[0].cpu().numpy().astype(np.float64)
    alpha = plan.k8_alpha[0].cpu().numpy().astype(np.float64)
    scale = plan.k8_scale[0].cpu().numpy().astype(np.float64)
    err_gpu = plan.k8_err[0].cpu().numpy().astype(np.float64)
    if centre:
        # the direction: the normalised sum of the unit blocks taken at even steps through the pool (up to 64 of them)
        n_s = min(P, 64)
        want_m = unit[[s * P // n_s for s in range(n_s)]].sum(0)
        want_m /= np.linalg.norm(want_m)
        assert np.abs(m - want_m).max() < 1e-6
        assert np.abs(alpha[live] - unit[live] @ m).max() < 1e-6
        if kind == "bf16_common":
            assert alpha[live].min() > 0.7              # the shared component is most of every block
    else:
        assert (m == 0).all() and (alpha == 0).all()
    assert (alpha[~live] == 0).all() and (scale > 0).all()
    uc = unit - alpha[:, None] * m[None]
    c = np.sqrt((uc ** 2).sum(1))
    assert np.abs(scale[live] * 256.0 / c[live] - 1.0).max() < 1e-4           # the scale follows |u_c| (it need not be exact)
    # every byte is a nearest e4m3 value of u_c / scale: spacing 2^(e - 3) at binade e, 2^-9 below 2^-6; the kernel
    # rounds the product to binary32 first, hence the small allowance
    target = np.where(live[:, None], uc / scale[:, None], 0.0)
    assert np.abs(target).max() < 448.0
    spacing = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(target), 2.0 ** -6))) - 3), 2.0 ** -9)
    assert (np.abs(dec - target) <= 0.5 * spacing * (1 + 1e-5)).all()
    # the stored error: the measured distance, plus a margin that covers what the identity <u, v> = <u_c, v_c> +
    # alpha_u alpha_v loses because the stored m and alpha are binary32 values (recomputed here: far below the margin)
    err_copy = np.sqrt(((uc - dec * scale[:, None]) ** 2).sum(1))
    loss = np.abs((uc * m[None]).sum(1)) + np.abs(alpha) * abs((m ** 2).sum() - 1.0)
    assert loss.max() < 5e-7
    err_true = np.where(live, err_copy + loss, 0.0)
    assert (err_gpu >= err_true + np.where(live, 2e-6, 0.0)).all() and (err_gpu <= err_copy * (1 + 2e-5) + 4e-6).all()
    assert (err_gpu[~live] == 0).all() and 0.002 < err_gpu[live].mean() < 0.04
    _say("fp8 copy", kind, "centred" if centre else "plain", "mean err", err_gpu[live].mean(), "max err", err_gpu.max(),
         "mean |u_c|", c[live].mean())
    L, R = bth[:ml], bth[ml:]
    S = oracle.similarity(Kh, nk, L, R)
    S_q = dense[0].cpu().numpy().reshape(ml, mr).astype(np.float64)
    ea, eb = err_gpu[L][:, None], err_gpu[R][None, :]
    slack = ea + eb + ea * eb + Kh.shape[1] * 2.0 ** -22
    worst = (np.abs(S_q - S) / slack).max()
    _say("  max |value - cos| / bound =", worst, "  mean bound", slack.mean())
    assert worst <= 1.0
    # and the value is what the decoded bytes give (format and operand layout of the matrix instruction)
    exact_q = (dec[L] * scale[L, None]) @ (dec[R] * scale[R, None]).T + alpha[L][:, None] * alpha[R][None, :]
    assert np.abs(S_q - exact_q).max() <= Kh.shape[1] * 2.0 ** -22
    if centre and kind == "bf16_common":
        assert slack.mean() < 0.03          # against about 0.05 uncentred: the intervals shrink with |u_c|


@pytest.mark.parametrize("centre", [False, True])
@pytest.mark.parametrize("rule", ["argmax", "first_row"])
@pytest.mark.parametrize("which", ["small_bf16", "small_bf16_cap2", "zipf_small", "zipf_at_threshold", "mixed_small_f32",
                                   "r4096_bf16_with_quarter_prefix", "tiny_f32_with_half_prefix", "r8192_bf16_long_blocks",
                                   "zipf_at_threshold_with_half_prefix", "small_bf16_cap2_with_half_prefix", "r128_bf16_two_slices"])
def test_tree_fp8_screen_gives_the_same_tables(kb, oracle, which, rule, centre):
    """The fp8 screen (similarity over one-byte copies of the key blocks + their measured error as a bound, every candidate
    evaluated in full in fp64) must give exactly the oracle's tables, pools and counters, alone and together with the prefix
    screen, for both pool types and both readings of the threshold line, with and without the common direction taken out
    of the copies (which the library only does where the prefix screen is off)."""
    kw = dict(rule=rule, screen_fp8="centred" if centre else True)
    if which == "small_bf16":
        rec = _small_bf16()
    elif which == "small_bf16_cap2":
        rec, kw = _small_bf16(n_req=5, tokens=900), dict(kw, cand_cap=2)
    elif which == "zipf_small":
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, thr=0.9)
        kw = dict(kw, cand_cap=8)
    elif which == "zipf_at_threshold":
        sigma = 0.05
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, sigma=sigma,
                          thr=1.0 / (1.0 + sigma * sigma))
    elif which == "mixed_small_f32":
        rec = wl.mixed(n_req=9, min_tokens=40, max_tokens=900, chunk_tokens=256, layers=1, kv_heads=2, pool=48, t=8, d=32,
                       dtype=torch.float32)
    elif which == "r4096_bf16_with_quarter_prefix":
        rec = wl.zipf_bff(n_req=6, tokens=32 * 150, layers=1, kv_heads=2, pool=400, t=32, d=128, thr=0.95)
        kw = dict(kw, screen_prefix=1024, cand_cap=8)
    elif which == "zipf_at_threshold_with_half_prefix":
        sigma = 0.05
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, sigma=sigma,
                          thr=1.0 / (1.0 + sigma * sigma))
        kw = dict(kw, screen_prefix=1024)
    elif which == "r128_bf16_two_slices":
        rec = _small_bf16(n_req=4, tokens=4 * 140, t=4, d=32, prefix_tokens=32)        # the shortest blocks the byte copies allow
    elif which == "small_bf16_cap2_with_half_prefix":
        rec, kw = _small_bf16(n_req=5, tokens=900), dict(kw, cand_cap=2, screen_prefix=128)
    elif which == "r8192_bf16_long_blocks":
        # blocks too long for a wavefront's registers: the norm pass, the merge step and the re-check take their streaming
        # forms, and the copies of rebuilt targets come from the kernel that follows the merge
        rec = wl.zipf_bff(n_req=5, tokens=64 * 30, layers=1, kv_heads=1, pool=40, t=64, d=128, thr=0.9)
        kw = dict(kw, band=2.5e-3)          # at least r * 2^-22
    else:
        rec, kw = wl.tiny_bff(), dict(kw, screen_prefix=512, cand_cap=4)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "fp8_screen_" + which + ("_centred" if centre else ""), **kw)
    assert stats.fused > 0
    centred_here = bool(centre) and not kw.get("screen_prefix") and rec.r <= 8192
    assert bool((plan.k8_alpha != 0).any()) == centred_here


_OVERFLOW_SEEN = {}


@pytest.mark.parametrize("screen", ["full", "prefix", "fp8", "both", "fp8_centred"])
def test_tree_screens_when_unrelated_blocks_share_a_direction(kb, oracle, screen):
    """Keys with a strong common component (unrelated blocks at cosine 0.8, threshold 0.9): the case the prefix screen and
    the plain byte copies are not made for.  Their bounds list many pairs that do not fuse, candidate lists overflow and
    columns are rescanned in fp64 -- slower, and still exactly the oracle's tables, pools and counters.  Copies with the
    common direction taken out keep their resolution here: far fewer columns overflow."""
    rec = _small_bf16(n_req=5, tokens=8 * 110, kv_heads=2)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(4242)
    for g in range(rec.G):
        mu = (2.0 * torch.randn(rec.r, generator=gen)).to(DEV)
        mat["K"][g] = (mat["K"][g].float() + mu).to(rec.dtype)
    host = gu.host_copy(mat)
    prefix = {"prefix": 64, "both": 128}.get(screen, 0)       # blocks of 256 elements; the byte copies need 128 at least
    fp8 = "centred" if screen == "fp8_centred" else screen in ("fp8", "both")
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, cand_cap=8, screen_prefix=prefix, screen_fp8=fp8)
    res = gu.oracle_fuse(oracle, rec, host)
    assert gu.check_ambiguity(res, "common_direction_" + screen) == list(range(rec.G))
    for g in range(rec.G):
        gu.compare_group(res[g], cache, g, False, "common_direction_" + screen)
    assert stats.fused == sum(int(r.stats[1]) for r in res) > 50
    assert stats.near_threshold == sum(int(r.stats[2]) for r in res)
    _say("  screen", screen, "fused", stats.fused, "refined", stats.refined, "overflow", stats.cand_overflow)
    _OVERFLOW_SEEN[screen] = stats.cand_overflow
    if screen not in ("full", "fp8_centred"):
        assert stats.cand_overflow > 0        # the bounds did list more pairs than the lists hold
    if screen == "fp8_centred" and "fp8" in _OVERFLOW_SEEN:
        assert stats.cand_overflow * 4 < _OVERFLOW_SEEN["fp8"]


@pytest.mark.parametrize("seed", list(range(20)))
def test_tree_seeded_sweep_with_a_common_direction(kb, oracle, seed):
    """Seeded variations of the case above: strength of the common component, threshold, pool type, candidate slots, both
    readings of the threshold line, all five screens.  Many of them overflow most candidate lists."""
    rng = np.random.default_rng(1000 + seed)
    dtype = torch.bfloat16 if seed % 3 else torch.float32
    rec = wl.llama8b_bff(n_req=int(rng.integers(3, 7)), tokens=8 * int(rng.integers(40, 120)), layers=1, kv_heads=2,
                         prefix_tokens=8 * int(rng.integers(0, 8)), near_pool=int(rng.integers(4, 30)), t=8, d=32, dtype=dtype,
                         seed=seed)
    rec.thr = float(rng.choice([0.8, 0.85, 0.9, 0.95]))
    mat = wl.materialise(rec, DEV, phys_perm=True)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    amp = float(rng.choice([0.5, 1.0, 2.0, 3.0]))
    for g in range(rec.G):
        mu = (amp * torch.randn(rec.r, generator=gen)).to(DEV)
        mat["K"][g] = (mat["K"][g].float() + mu).to(rec.dtype)
    host = gu.host_copy(mat)
    screen = ("full", "prefix", "fp8", "both", "fp8_centred")[seed % 5]
    rule = "first_row" if (seed // 5) % 2 else "argmax"
    prefix = {"prefix": 64, "both": 128}.get(screen, 0)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, cand_cap=int(rng.choice([2, 8, 64])), rule=rule, screen_prefix=prefix,
                                          screen_fp8="centred" if screen == "fp8_centred" else screen in ("fp8", "both"))
    res = gu.oracle_fuse(oracle, rec, host, rule=rule)
    assert gu.check_ambiguity(res, f"common_direction_sweep_{seed}") == list(range(rec.G))
    for g in range(rec.G):
        gu.compare_group(res[g], cache, g, rec.dtype == torch.float32, f"common_direction_sweep_{seed}")
    assert stats.fused == sum(int(r.stats[1]) for r in res) and stats.near_threshold == sum(int(r.stats[2]) for r in res)
    _say("  seed", seed, screen, rule, "amp", amp, "thr", rec.thr, "fused", stats.fused, "refined", stats.refined, "overflow",
         stats.cand_overflow)


@pytest.mark.parametrize("centre", [False, True])
def test_fp8_screen_step_by_step_and_arguments(kb, oracle, centre):
    """The single-step entry points with the fp8 screen on (the copy then comes from kvfuse_leaf_sets and is refreshed after
    every kvfuse_merge), once together with the prefix screen and once with centred copies, and the argument checks of the
    switch."""
    rec = _small_bf16(n_req=5, tokens=1000, kv_heads=2)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    host = gu.host_copy(mat)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr), 16)
    k8 = torch.empty(cache.G, cache.P, rec.r, device=DEV, dtype=torch.uint8)
    err = torch.empty(3 * cache.G * cache.P + cache.G * rec.r, device=DEV, dtype=torch.float32)
    # one of the two arrays missing
    assert kb.lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, k8.data_ptr(), k8.numel(), None, 0, 0) == kb.EINVAL
    assert kb.lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, None, 0, err.data_ptr(), err.numel(), 0) == kb.EINVAL
    # arrays smaller than the copies and their side values need
    assert kb.lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, k8.data_ptr(), k8.numel() - 1, err.data_ptr(), err.numel(), 0) == kb.EINVAL
    assert kb.lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, k8.data_ptr(), k8.numel(), err.data_ptr(), cache.G * cache.P, 1) == kb.EINVAL
    # a prefix that is fine for the bfloat16 product (96 elements = 192 bytes of the pool) is no multiple of 64 bytes of the copy
    kb.set_screen_prefix(ctx, plan, 96)
    assert kb.lib.kvfuse_plan_set_screen_fp8(ctx.h, plan.h, k8.data_ptr(), k8.numel(), err.data_ptr(), err.numel(), 0) == kb.EINVAL
    kb.set_screen_prefix(ctx, plan, 0)
    kb.set_screen_fp8(ctx, plan, centre=centre)
    with pytest.raises(kb.KvfuseError):
        kb.set_screen_prefix(ctx, plan, 96)
    if not centre:
        kb.set_screen_prefix(ctx, plan, 128)
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)
    for h in range(plan.n_heights):
        kb.similarity(ctx, plan, h, rec.thr)
        kb.assign(ctx, plan, h, rec.thr)
        kb.merge(ctx, plan, h)
    kb.rewrite_block_table(ctx, cache)
    torch.cuda.synchronize()
    res = gu.oracle_fuse(oracle, rec, host)
    assert gu.check_ambiguity(res, "fp8_step_by_step") == list(range(rec.G))
    for g in range(rec.G):
        gu.compare_group(res[g], cache, g, False, "fp8_step_by_step")
    assert sum(int(r.stats[1]) for r in res) > 50
    assert bool((plan.k8_alpha != 0).any()) == centre
    # blocks too short or of an odd length for the byte copy
    small = wl.tiny_bff()
    m2 = wl.materialise(small, DEV)
    c2 = kb.Cache(m2["K"][:, :, :96].contiguous(), m2["V"][:, :, :96].contiguous(), m2["bt"], 4, 24)
    p2 = kb.Plan(ctx, c2, kb.tree_spec(small.leaf_start, small.leaf_count, small.unit_leaf_ptr), 4)
    with pytest.raises(kb.KvfuseError):
        kb.set_screen_fp8(ctx, p2)


def test_prefix_screen_rejects_bad_arguments(kb):
    rec = _small_bf16()
    mat = wl.materialise(rec, DEV)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr))
    for bad in (rec.r, rec.r + 32, 32, 48, -64):      # whole block or more, one slice, not whole slices, negative
        with pytest.raises(kb.KvfuseError) as e:
            kb.set_screen_prefix(ctx, plan, bad)
        assert e.value.code == kb.EINVAL
    assert kb.lib.kvfuse_plan_set_screen_prefix(ctx.h, plan.h, 64, None) == kb.EINVAL      # no tail-share array
    kb.set_screen_prefix(ctx, plan, 64)
    kb.set_screen_prefix(ctx, plan, 0)


@pytest.mark.parametrize("cand_cap", [16, 2])
@pytest.mark.parametrize("which", ["zipf_small", "small_bf16", "mixed_small_f32", "zipf_at_threshold"])
def test_tree_first_row_rule(kb, oracle, which, cand_cap):
    """Algorithm 1's row loop taken literally (the lowest row above the threshold takes the block), on inputs where
    many right blocks clear the threshold for several left rows; two candidate slots force the full-column path."""
    if which == "zipf_small":
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, thr=0.9)
    elif which == "zipf_at_threshold":
        # two noisy copies base + N(0, sigma) of one base have cosine 1 / (1 + sigma^2) up to O(sigma^2 / sqrt(r)): with
        # the threshold there, most listed rows are undecided by the screen and the fp64 re-check walks them in row order
        sigma = 0.05
        rec = wl.zipf_bff(n_req=8, tokens=32 * 40, layers=1, kv_heads=2, pool=60, t=32, d=64, sigma=sigma,
                          thr=1.0 / (1.0 + sigma * sigma))
    elif which == "small_bf16":
        rec = _small_bf16()
    else:
        rec = wl.mixed(n_req=9, min_tokens=40, max_tokens=900, chunk_tokens=256, layers=1, kv_heads=2, pool=48, t=8, d=32,
                       dtype=torch.float32)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, which + "_first_row", cand_cap=cand_cap, rule="first_row")
    if which == "zipf_at_threshold":
        assert stats.refined > 100 and stats.near_threshold > 100
        if cand_cap == 16:
            assert stats.cand_overflow < stats.refined
    # the case has power only if the two readings disagree somewhere
    other = gu.oracle_fuse(oracle, rec, gu.host_copy(wl.materialise(rec, DEV, phys_perm=True)))
    differ = sum(int((a.bt != b.bt).sum()) for a, b in zip(res, other))
    _say("  logical blocks whose target differs between the two readings:", differ)
    if which != "small_bf16":
        assert differ > 0
    assert sum(r.n_physical for r in res) == stats.physical_blocks


@pytest.mark.parametrize("which", ["mixed_small", "bff_ragged_lengths", "cff_short_tail"])
def test_tree_shortest_first_order(kb, oracle, which):
    """Remark on the order of requests: the tree is built over the units in ascending number of blocks while the
    table keeps its layout, so leaves are no longer in logical order."""
    if which == "mixed_small":
        rec = wl.mixed(n_req=9, min_tokens=40, max_tokens=900, chunk_tokens=256, layers=1, kv_heads=2, pool=48, t=8, d=32)
    elif which == "bff_ragged_lengths":
        rec = wl.mixed(n_req=7, min_tokens=64, max_tokens=1500, chunk_tokens=1 << 20, layers=1, kv_heads=2, pool=40, t=8, d=32)
    else:
        rec = wl.cff_long(tokens=8 * 580, chunk_tokens=8 * 75, layers=1, kv_heads=2, t=8, d=32)
    spec = kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.group_size)
    new_spec, order = kb.tree_spec_shortest_first(spec)
    ls, lc, up, want = oracle.shortest_first(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr)
    assert order.tolist() == want.tolist() and order.tolist() != sorted(order.tolist())
    assert np.array_equal(np.ctypeslib.as_array((C.c_int32 * len(ls)).from_address(new_spec.leaf_start)), ls)
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, which + "_shortest_first", shortest_first=True)
    given = gu.oracle_fuse(oracle, rec, gu.host_copy(wl.materialise(rec, DEV, phys_perm=True)))
    _say("  physical blocks: given order", sum(r.n_physical for r in given), "shortest first", stats.physical_blocks)
    assert stats.fused > 20


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6, 10, 14, 20, 21, 22, 23, 24, 25, 27, 30, 33, 35])
def test_tree_seeded_sweep(kb, oracle, seed):
    """Seeded small workloads of all four structures with the variants mixed at random: assignment rule, request order,
    request groups, candidate slots (1 slot = every multi-candidate column is rescanned), dtype, and which screen the
    similarity step uses (full product, prefix, fp8 copies, both)."""
    rng = np.random.default_rng(seed)
    kind = seed % 4
    dtype = torch.bfloat16 if seed % 3 else torch.float32
    if kind == 0:
        rec = wl.llama8b_bff(n_req=int(rng.integers(2, 9)), tokens=8 * int(rng.integers(20, 160)), layers=1, kv_heads=2,
                             prefix_tokens=8 * int(rng.integers(0, 12)), near_pool=int(rng.integers(4, 40)), t=8, d=32,
                             dtype=dtype, seed=seed)
    elif kind == 1:
        rec = wl.mixed(n_req=int(rng.integers(3, 12)), min_tokens=20, max_tokens=int(rng.integers(200, 1200)),
                       chunk_tokens=int(rng.choice([128, 256, 512])), layers=1, kv_heads=2, pool=int(rng.integers(8, 60)),
                       t=8, d=32, dtype=dtype, seed=seed)
    elif kind == 2:
        rec = wl.zipf_bff(n_req=int(rng.integers(3, 10)), tokens=16 * int(rng.integers(10, 50)), layers=1, kv_heads=2,
                          pool=int(rng.integers(10, 80)), t=16, d=32, sigma=float(rng.choice([0.03, 0.05, 0.2])),
                          thr=float(rng.choice([0.85, 0.9, 0.97, 0.9975])), dtype=dtype, seed=seed)
    else:
        rec = wl.cff_long(tokens=8 * int(rng.integers(200, 700)), chunk_tokens=8 * int(rng.integers(30, 100)), layers=1,
                          kv_heads=2, t=8, d=32, dtype=dtype, seed=seed)
    rule = "first_row" if seed % 2 else "argmax"
    shortest_first = bool(seed % 5 == 0 or seed % 7 == 0)
    group_size = int(rng.choice([0, 0, 2, 3]))
    cand_cap = int(rng.choice([1, 3, 16, 64]))
    screen = ("full", "prefix", "fp8", "both")[(seed // 2) % 4]      # blocks have 256 or 512 elements here
    _run_tree_case(kb, oracle, rec, f"sweep_{seed}_{screen}", cand_cap=cand_cap, rule=rule, shortest_first=shortest_first,
                   group_size=group_size, screen_prefix=128 if screen in ("prefix", "both") else 0,
                   screen_fp8=screen in ("fp8", "both"))


def test_tree_variants_combined(kb, oracle):
    """Row-order rule, shortest-first tree and "every N requests" together, on ragged chunked requests in f32 and bf16."""
    for dtype, gs in ((torch.float32, 4), (torch.bfloat16, 3)):
        rec = wl.mixed(n_req=10, min_tokens=40, max_tokens=800, chunk_tokens=256, layers=1, kv_heads=2, pool=40, t=8, d=32,
                       dtype=dtype)
        cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, f"variants_combined_{gs}", cand_cap=4, rule="first_row",
                                                      shortest_first=True, group_size=gs)
        assert stats.fused > 20


@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_replicate_rescaled_and_drop_rescale_match_oracle(kb, oracle, kind):
    """The two evaluation modes of the results section.  Replicate: every logical block gets the block it had before
    fusion back, holding scale * representative in the pool type (bit-exact against the oracle), the table returns to
    the original one, and plain decode attention over the result agrees with the oracle's.  Drop: unit scales."""
    rec = wl.llama8b_bff(n_req=5, tokens=16 * 60, layers=1, kv_heads=2, prefix_tokens=96, near_pool=16, t=16, d=64,
                         dtype=torch.bfloat16 if kind == "bf16" else torch.float32)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    host = gu.host_copy(mat)
    bt0 = mat["bt"].clone()
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    res = gu.oracle_fuse(oracle, rec, host)
    assert stats.fused > 20 and stats.fused == sum(int(r.stats[1]) for r in res)
    for g in range(rec.G):
        gu.compare_group(res[g], cache, g, kind == "f32", "replicate/fused")
    # drop-rescale on a copy of the table state: scales become one, nothing else moves
    sk, sv, btf = cache.scale_k.clone(), cache.scale_v.clone(), cache.bt.clone()
    kb.drop_rescale(ctx, cache)
    torch.cuda.synchronize()
    assert (cache.scale_k == 1).all() and (cache.scale_v == 1).all() and torch.equal(cache.bt, btf)
    assert not (sk == 1).all()
    cache.scale_k.copy_(sk)
    cache.scale_v.copy_(sv)
    # replicate
    _say("replicate", kind, "G", rec.G, "n", rec.n, "fused", stats.fused)
    kb.replicate_rescaled(ctx, cache, bt0)
    torch.cuda.synchronize()
    assert torch.equal(cache.bt, bt0)
    assert (cache.scale_k == 1).all() and (cache.scale_v == 1).all() and (cache.remap == -1).all()
    Kr, Vr = [], []
    for g in range(rec.G):
        Kr.append(oracle.replicate_rescaled(res[g].kpool, host[2][g], res[g].bt, res[g].scale_k))
        Vr.append(oracle.replicate_rescaled(res[g].vpool, host[2][g], res[g].bt, res[g].scale_v))
        assert np.array_equal(wl.to_numpy_pool(cache.K[g]), Kr[g]), f"group {g}: replicated K differs"
        assert np.array_equal(wl.to_numpy_pool(cache.V[g]), Vr[g]), f"group {g}: replicated V differs"
        assert np.array_equal(cache.refcount[g].cpu().numpy(), np.bincount(host[2][g], minlength=cache.P))
        np.testing.assert_allclose(cache.norm_k[g].cpu().numpy(), oracle.block_norms(Kr[g]), rtol=1e-13)
        np.testing.assert_allclose(cache.orig_norm_v[g].cpu().numpy(), oracle.block_norms(Vr[g])[host[2][g]], rtol=1e-13)
    q = wl.queries(rec, DEV)
    out = _decode(kb, ctx, rec, cache, q)
    one = np.ones((rec.G, rec.n))
    want = oracle.paged_decode_attention(q[0].float().cpu().numpy().astype(np.float64), Kr, Vr, host[2], one, one,
                                         rec.req_start, rec.ctx_len, rec.t, rec.d)
    err = np.abs(out[0] - want).max() / np.abs(want).max()
    _say("  decode over the replicated cache: max rel err", err)
    assert err < (2e-3 if kind == "bf16" else 1e-5)


def test_variant_entry_points_reject_bad_arguments(kb):
    rec = wl.tiny_bff()
    mat = wl.materialise(rec, DEV)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, 0), 16)
    with pytest.raises(kb.KvfuseError):
        kb.set_assign_rule(ctx, plan, 7)
    with pytest.raises(kb.KvfuseError):
        ctx.check(kb.lib.kvfuse_replicate_rescaled(ctx.h, C.byref(cache.pool), C.byref(cache.table), None))
    # overlapping leaves are refused whatever their order; disjoint leaves in any order are accepted
    with pytest.raises(kb.KvfuseError):
        kb.Plan(ctx, cache, kb.tree_spec([8, 0, 4], [8, 8, 8], [0, 1, 2, 3], 0), 16)
    kb.Plan(ctx, cache, kb.tree_spec([16, 0, 8], [8, 8, 8], [0, 1, 2, 3], 0), 16)


@pytest.mark.parametrize("shape", ["r4096_bf16", "r8192_bf16", "r2048_f32", "r16384_bf16_all_heads", "r8192_f32"])
def test_tree_long_blocks(kb, oracle, shape):
    """Block lengths beyond the bench shape: config 4's 32 x 128 blocks (8 KiB rows: 128 K-slices per row in the
    similarity kernels, two-wavefront merge items), the longest supported block (t*d = 8192: workgroup-per-target
    merge) and binary32 blocks of 8 KiB.  Sets are large enough for the 256 x 256 tiles at the upper heights."""
    if shape == "r4096_bf16":
        rec = wl.zipf_bff(n_req=6, tokens=32 * 150, layers=1, kv_heads=2, pool=400, t=32, d=128, thr=0.9)
    elif shape == "r8192_bf16":
        rec = wl.zipf_bff(n_req=4, tokens=64 * 90, layers=1, kv_heads=1, pool=200, t=64, d=128, thr=0.9)
    elif shape == "r16384_bf16_all_heads":
        # the paper's own vector: one per block over all 8 KV heads of a layer (t = 16, h * d = 1024), one table per
        # layer -- for the fusion steps simply a pool with G = layers and d := h * d
        rec = wl.zipf_bff(n_req=4, tokens=16 * 90, layers=2, kv_heads=1, pool=200, t=16, d=1024, thr=0.9)
    elif shape == "r8192_f32":
        rec = wl.zipf_bff(n_req=3, tokens=64 * 100, layers=1, kv_heads=1, pool=150, t=64, d=128, thr=0.9, dtype=torch.float32)
    else:
        rec = wl.zipf_bff(n_req=4, tokens=16 * 150, layers=1, kv_heads=1, pool=300, t=16, d=128, thr=0.9, dtype=torch.float32)
    # the screen's error bound grows with the block length: the band must be at least r * 2^-22
    cache, plan, stats, res, mat = _run_tree_case(kb, oracle, rec, "long_blocks_" + shape, cand_cap=8,
                                                  band=max(1e-3, 1.25 * rec.r * 2.0 ** -22))
    assert stats.fused > 50
    if rec.d > 128:
        return                      # the attention kernels need the per-head layout
    q = wl.queries(rec, DEV)
    out = _decode(kb, ctx=kb.Context(DEV), rec=rec, cache=cache, q=q)
    ref = _attn_oracle(oracle, rec, cache, q[0], 0, rec.kv_heads)
    assert np.abs(out[0] - ref).max() <= (1e-4 if rec.dtype == torch.float32 else 5e-3)


def _direct_case(kb, oracle, K, V, leaf_start, leaf_count, unit_leaf_ptr, thr, name, t=8, d=32, cand_cap=16, rule="argmax"):
    """Pools given as float arrays [G][n][r]; identity table.  Runs both sides and compares every group exactly."""
    G, n, r = K.shape
    assert r == t * d
    dt = torch.bfloat16
    Kd = torch.from_numpy(K).to(DEV).to(dt).contiguous()
    Vd = torch.from_numpy(V).to(DEV).to(dt).contiguous()
    bt = torch.arange(n, dtype=torch.int32, device=DEV).repeat(G, 1).contiguous()
    Kh = [wl.to_numpy_pool(Kd[g]) for g in range(G)]
    Vh = [wl.to_numpy_pool(Vd[g]) for g in range(G)]
    _say("direct case", name, "G", G, "n", n, "leaves", list(leaf_count))
    ctx = kb.Context(DEV)
    cache = kb.Cache(Kd, Vd, bt, t, d)
    plan = kb.Plan(ctx, cache, kb.tree_spec(leaf_start, leaf_count, unit_leaf_ptr, 0), cand_cap)
    if rule != "argmax":
        kb.set_assign_rule(ctx, plan, kb.RULE_FIRST_ROW)
    stats = kb.fuse_tree(ctx, plan, thr, want_stats=True)
    torch.cuda.synchronize()
    res = [oracle.fuse_group(Kh[g], Vh[g], np.arange(n, dtype=np.int32), leaf_start, leaf_count, unit_leaf_ptr, thr, rule=rule)
           for g in range(G)]
    for g in range(G):
        gu.compare_group(res[g], cache, g, False, name)
    assert stats.fused == sum(int(x.stats[1]) for x in res)
    return cache, plan, stats, res


def test_tree_degenerate_inputs(kb, oracle):
    """Edges of the input space: one leaf (no tree at all), empty leaves and an empty unit among real ones, a table
    with no leaves, every block identical (all cosines exactly 1: every decision is a tie between all left rows and
    goes to the lowest), an all-zero pool (zero blocks never fuse), and two identical requests (the right one vanishes)."""
    rng = np.random.default_rng(77)
    t, d, G = 8, 32, 2
    r = t * d
    # one request, one leaf: nothing to compare
    K = rng.standard_normal((G, 12, r)).astype(np.float32)
    V = rng.standard_normal((G, 12, r)).astype(np.float32)
    cache, plan, stats, res = _direct_case(kb, oracle, K, V, [0], [12], [0, 1], 0.5, "one_leaf")
    assert plan.n_heights == 0 and stats.fused == 0 and stats.compression_ratio == 1.0
    # no leaves at all: norms and table initialisation only
    cache, plan, stats, res = _direct_case(kb, oracle, K, V, [], [], [0], 0.5, "no_leaves")
    assert stats.fused == 0 and (cache.refcount == 1).all()
    # empty leaves and an empty unit between real ones (units: [leaf0], [], [leaf1(empty), leaf2], [leaf3])
    K = np.tile(rng.standard_normal((1, 5, r)).astype(np.float32), (G, 3, 1))[:, :12] + \
        0.02 * rng.standard_normal((G, 12, r)).astype(np.float32)
    V = rng.standard_normal((G, 12, r)).astype(np.float32)
    cache, plan, stats, res = _direct_case(kb, oracle, K, V, [0, 4, 4, 8], [4, 0, 4, 4], [0, 1, 1, 3, 4], 0.9, "empty_leaves")
    assert stats.fused > 0
    # every block identical
    one = rng.standard_normal((1, 1, r)).astype(np.float32)
    K = np.tile(one, (G, 20, 1))
    V = np.tile(one[:, :, ::-1], (G, 20, 1))
    for rule in ("argmax", "first_row"):
        cache, plan, stats, res = _direct_case(kb, oracle, K, V, [0, 5, 10, 15], [5, 5, 5, 5], [0, 1, 2, 3, 4], 0.9,
                                               "all_identical_" + rule, cand_cap=4, rule=rule)
        assert stats.fused == G * 15
        if rule == "first_row":
            assert (cache.bt[:, 5:] == 0).all() and (cache.refcount[:, 0] == 16).all()
        else:
            # at the top node the raw blocks 11 .. 14 are exactly equal to the raw left rows 1 .. 4 but only almost
            # equal to row 0, which by then holds a rounded representative: the most similar row is row 1
            assert (cache.bt[:, 11:15] == 1).all() and (cache.bt[:, 5:11] == 0).all() and (cache.bt[:, 15:] == 0).all()
    # all-zero pool
    Z = np.zeros((G, 16, r), np.float32)
    cache, plan, stats, res = _direct_case(kb, oracle, Z, Z, [0, 8], [8, 8], [0, 1, 2], 0.0, "all_zero")
    assert stats.fused == 0 and (cache.scale_k == 1).all() and (cache.norm_k == 0).all()
    # two identical requests, random inside: block j of the right one goes to block j of the left one
    half = rng.standard_normal((G, 9, r)).astype(np.float32)
    K = np.concatenate([half, half], 1)
    V = np.concatenate([half[:, :, ::-1], half[:, :, ::-1]], 1).copy()
    cache, plan, stats, res = _direct_case(kb, oracle, K, V, [0, 9], [9, 9], [0, 1, 2], 0.99, "twin_requests")
    assert stats.fused == G * 9 and torch.equal(cache.bt[:, 9:], cache.bt[:, :9]) and stats.compression_ratio == 2.0


def test_decode_empty_and_minimal_requests(kb, oracle):
    """Requests with no context, with one token, and a call with no request at all."""
    rng = np.random.default_rng(78)
    t, d, H, Hq = 16, 64, 2, 8
    ctx_len = np.array([0, 1, 16, 17, 0, 40], np.int32)
    blocks = np.maximum((ctx_len + t - 1) // t, 0)
    req_start = np.concatenate([[0], np.cumsum(blocks)[:-1]]).astype(np.int32)
    n = max(int(blocks.sum()), 1)
    Kd = torch.from_numpy(rng.standard_normal((H, n, t * d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    Vd = torch.from_numpy(rng.standard_normal((H, n, t * d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    bt = torch.arange(n, dtype=torch.int32, device=DEV).repeat(H, 1).contiguous()
    ctx = kb.Context(DEV)
    cache = kb.Cache(Kd, Vd, bt, t, d)
    cache.identity_scales()
    q = torch.from_numpy(rng.standard_normal((1, len(ctx_len), Hq, d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    rs = torch.tensor(req_start, dtype=torch.int32, device=DEV)
    cl = torch.tensor(ctx_len, dtype=torch.int32, device=DEV)
    out = kb.paged_decode_attn(ctx, cache, H, q, rs, cl, int(blocks.max()))
    torch.cuda.synchronize()
    one = np.ones((H, n))
    want = oracle.paged_decode_attention(q[0].float().cpu().numpy().astype(np.float64), [wl.to_numpy_pool(Kd[g]) for g in range(H)],
                                         [wl.to_numpy_pool(Vd[g]) for g in range(H)], [np.arange(n)] * H, one, one, req_start,
                                         ctx_len, t, d)
    got = out[0].cpu().numpy()
    assert np.abs(got - want).max() <= 5e-3
    assert (got[0] == 0).all() and (got[4] == 0).all()                      # no context: zero output, not NaN
    assert np.allclose(got[1], np.repeat(Vd[:, req_start[1], :d].float().cpu().numpy(), Hq // H, 0), atol=1e-6)   # one token: its value
    # no request at all
    q0 = torch.empty(1, 0, Hq, d, device=DEV, dtype=torch.bfloat16)
    out0 = kb.paged_decode_attn(ctx, cache, H, q0, rs[:0], cl[:0], 0)
    torch.cuda.synchronize()
    assert out0.shape == (1, 0, Hq, d)


def test_tree_is_deterministic(kb):
    rec = _small_bf16(n_req=5, tokens=480, kv_heads=2)
    outs = []
    for _ in range(2):
        mat = wl.materialise(rec, DEV, phys_perm=True)
        cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
        outs.append((cache.bt.clone(), cache.K.clone(), cache.V.clone(), cache.scale_k.clone(), cache.refcount.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_bad_arguments_are_reported_not_crashed(kb):
    rec = wl.tiny_bff()
    mat = wl.materialise(rec, DEV)
    ctx = kb.Context(DEV)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    with pytest.raises(kb.KvfuseError) as e:
        kb.Plan(ctx, cache, kb.tree_spec([0, 4], [8, 8], [0, 1, 2]))        # overlapping leaves
    assert e.value.code == kb.EINVAL
    plan = kb.Plan(ctx, cache, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr))
    with pytest.raises(kb.KvfuseError) as e:
        kb.similarity(ctx, plan, 7, 0.9)                                    # no such height
    assert e.value.code == kb.EINVAL
    with pytest.raises(kb.KvfuseError) as e:
        kb.fuse_tree(ctx, plan, 0.9, band=1e-9)                             # band below the screen's error bound
    assert e.value.code == kb.EINVAL
    bad = kb.Cache(mat["K"][:, :, :1000].contiguous(), mat["V"][:, :, :1000].contiguous(), mat["bt"], 8, 125)
    with pytest.raises(kb.KvfuseError) as e:
        kb.block_norms(ctx, bad)                                            # block bytes not a multiple of 128
    assert e.value.code == kb.ESHAPE
    # an id outside the pool is clamped inside the kernels and reported by the pipeline
    mat2 = wl.materialise(rec, DEV)
    mat2["bt"][0, 3] = 10 ** 6
    cache2 = kb.Cache(mat2["K"], mat2["V"], mat2["bt"], rec.t, rec.d)
    plan2 = kb.Plan(ctx, cache2, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr))
    with pytest.raises(kb.KvfuseError) as e:
        kb.fuse_tree(ctx, plan2, 0.95)
    assert e.value.code == kb.EINVAL
    torch.cuda.synchronize()
    # a table that already shares a block (a second fusion over a fused table, a prefix cache) is refused as well:
    # Algorithm 1 starts from unshared blocks
    mat3 = wl.materialise(rec, DEV)
    mat3["bt"][1, 20] = mat3["bt"][1, 2]
    cache3 = kb.Cache(mat3["K"], mat3["V"], mat3["bt"], rec.t, rec.d)
    plan3 = kb.Plan(ctx, cache3, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr))
    with pytest.raises(kb.KvfuseError) as e:
        kb.fuse_tree(ctx, plan3, 0.95)
    assert e.value.code == kb.EINVAL and "not injective" in str(e.value)
    torch.cuda.synchronize()
    # key blocks whose products would leave binary32's range in the screen (here two copies of one block scaled by 2^-60,
    # which the fp64 oracle would fuse and a binary32 product cannot see) are reported, not silently mishandled
    mat4 = wl.materialise(rec, DEV)
    mat4["K"][0, 5] = mat4["K"][0, 5] * 2.0 ** -60
    mat4["K"][0, 20] = mat4["K"][0, 5]
    cache4 = kb.Cache(mat4["K"], mat4["V"], mat4["bt"], rec.t, rec.d)
    plan4 = kb.Plan(ctx, cache4, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr))
    with pytest.raises(kb.KvfuseError) as e:
        kb.fuse_tree(ctx, plan4, 0.95)
    assert e.value.code == kb.EINVAL and "2^-40" in str(e.value)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------ a7 decode attention

def _attn_oracle(oracle, rec, cache, q, layer, H):
    gs = [layer * H + h for h in range(H)]
    Kp = [wl.to_numpy_pool(cache.K[g]) for g in gs]
    Vp = [wl.to_numpy_pool(cache.V[g]) for g in gs]
    bt = [cache.bt[g].cpu().numpy() for g in gs]
    sk = [cache.scale_k[g].cpu().numpy().astype(np.float64) for g in gs]
    sv = [cache.scale_v[g].cpu().numpy().astype(np.float64) for g in gs]
    qh = q.float().cpu().numpy().astype(np.float64)
    return oracle.paged_decode_attention(qh, Kp, Vp, bt, sk, sv, rec.req_start, rec.ctx_len, rec.t, rec.d)


def _decode(kb, ctx, rec, cache, q):
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=DEV)
    cl = torch.tensor(rec.ctx_len, dtype=torch.int32, device=DEV)
    mb = int(((rec.ctx_len + rec.t - 1) // rec.t).max())
    out = kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, mb)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


def test_decode_tiny_config_fused_and_unfused(kb, oracle):
    """Config 1's four decode queries: after fusion, and with thr > 1 where attention must equal unfused paged
    attention (same kernel on the untouched table) bit for bit."""
    rec = wl.tiny_bff()
    q = wl.queries(rec, DEV)
    mat = wl.materialise(rec, DEV)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    out = _decode(kb, ctx, rec, cache, q)
    ref = _attn_oracle(oracle, rec, cache, q[0], 0, rec.kv_heads)
    err = np.abs(out[0] - ref).max()
    _say("decode tiny fused: max abs err", err)
    assert err <= 2e-2 and err <= 1e-4
    mat1 = wl.materialise(rec, DEV)
    cache1, plan1, stats1, ctx1 = gu.gpu_fuse(rec, mat1, thr=1.5)
    out1 = _decode(kb, ctx1, rec, cache1, q)
    mat2 = wl.materialise(rec, DEV)
    cache2 = kb.Cache(mat2["K"], mat2["V"], mat2["bt"], rec.t, rec.d)
    cache2.identity_scales()
    out2 = _decode(kb, ctx1, rec, cache2, q)
    assert np.array_equal(out1, out2)
    ref2 = _attn_oracle(oracle, rec, cache2, q[0], 0, rec.kv_heads)
    assert np.abs(out2[0] - ref2).max() <= 1e-4


@pytest.mark.parametrize("case", ["bf16_d128_gqa4", "bf16_d64_gqa8_t32", "bf16_split_long", "f32_d128_ragged"])
def test_decode_matches_oracle(kb, oracle, case):
    _say("decode case", case)
    if case == "bf16_d128_gqa4":
        rec = wl.llama8b_bff(n_req=5, tokens=16 * 37, layers=2, kv_heads=2, prefix_tokens=64, near_pool=16)
    elif case == "bf16_d64_gqa8_t32":
        rec = wl.zipf_bff(n_req=4, tokens=32 * 9, layers=1, kv_heads=2, pool=30, t=32, d=64)
    elif case == "bf16_split_long":
        rec = wl.cff_long(tokens=16 * 700, chunk_tokens=16 * 100, layers=1, kv_heads=2)
    else:
        rec = wl.mixed(n_req=6, min_tokens=20, max_tokens=700, chunk_tokens=256, layers=1, kv_heads=2, pool=40,
                       dtype=torch.float32)
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    assert stats.fused > 0
    q = wl.queries(rec, DEV)
    out = _decode(kb, ctx, rec, cache, q)
    worst = 0.0
    for layer in range(rec.layers):
        ref = _attn_oracle(oracle, rec, cache, q[layer], layer, rec.kv_heads)
        worst = max(worst, float(np.abs(out[layer] - ref).max()))
    _say("  max abs err", worst)
    assert worst <= 2e-2
    assert worst <= (1e-4 if rec.dtype == torch.float32 else 5e-3)


@pytest.mark.parametrize("case", ["bf16_h4_d128_gqa2", "bf16_h2_d64_gqa8_t32", "f32_h2_d64_split"])
def test_decode_through_all_head_blocks_matches_oracle(kb, oracle, case):
    """The paper's own vector (method section: r = t * h * d, one table per layer): fusion over all-head blocks, then
    decode attention through the per-layer table with kvfuse_paged_decode_attn_all_heads.  The oracle sees the same
    cache as H per-head pools that are strided views of the all-head pool and share the layer's table and scales."""
    _say("all-head decode case", case)
    if case == "bf16_h4_d128_gqa2":
        H, hd, rep, kw = 4, 128, 2, dict(n_req=5, tokens=16 * 40, layers=2, pool=80, t=16)
    elif case == "bf16_h2_d64_gqa8_t32":
        H, hd, rep, kw = 2, 64, 8, dict(n_req=4, tokens=32 * 25, layers=1, pool=40, t=32)
    else:
        H, hd, rep, kw = 2, 64, 2, dict(n_req=2, tokens=16 * 300, layers=1, pool=60, t=16, dtype=torch.float32)
    rec = wl.zipf_bff(kv_heads=1, d=H * hd, thr=0.9, **kw)        # for the fusion steps: G = layers, d := h * d
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, band=max(1e-3, 1.25 * rec.r * 2.0 ** -22))
    assert stats.fused > 0
    Hq = H * rep
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.MASTER_SEED + 11)
    q = torch.randn(rec.layers, rec.B, Hq, hd, generator=gen).to(rec.dtype).to(DEV)
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=DEV)
    cl = torch.tensor(rec.ctx_len - 5, dtype=torch.int32, device=DEV)          # a partial last block
    mb = int(rec.req_blocks.max())
    out = kb.paged_decode_attn_all_heads(ctx, cache, H, q, rs, cl, mb)
    torch.cuda.synchronize()
    worst = 0.0
    for layer in range(rec.layers):
        Kl = wl.to_numpy_pool(cache.K[layer]).reshape(rec.n, rec.t, H, hd)
        Vl = wl.to_numpy_pool(cache.V[layer]).reshape(rec.n, rec.t, H, hd)
        Kp = [np.ascontiguousarray(Kl[:, :, h, :]).reshape(rec.n, rec.t * hd) for h in range(H)]
        Vp = [np.ascontiguousarray(Vl[:, :, h, :]).reshape(rec.n, rec.t * hd) for h in range(H)]
        bt = [cache.bt[layer].cpu().numpy()] * H
        sk = [cache.scale_k[layer].cpu().numpy().astype(np.float64)] * H
        sv = [cache.scale_v[layer].cpu().numpy().astype(np.float64)] * H
        ref = oracle.paged_decode_attention(q[layer].float().cpu().numpy().astype(np.float64), Kp, Vp, bt, sk, sv, rec.req_start,
                                            rec.ctx_len - 5, rec.t, hd)
        worst = max(worst, float(np.abs(out[layer].cpu().numpy() - ref).max()))
    _say("  max abs err", worst)
    assert worst <= 2e-2
    assert worst <= (1e-4 if rec.dtype == torch.float32 else 5e-3)
    with pytest.raises(kb.KvfuseError) as e:                                     # query heads that the KV heads do not divide
        kb.paged_decode_attn_all_heads(ctx, cache, H, q[:, :, :Hq - 1].contiguous(), rs, cl, mb)
    assert e.value.code == kb.EINVAL


# ------------------------------------------------------------------------------------------ shared-block decode attention

def _decode_shared(kb, ctx, rec, cache, q, min_cluster_blocks):
    plan = kb.SharedDecodePlan(ctx, cache, rec.kv_heads, rec.req_start, rec.ctx_len, rec.q_heads,
                               min_cluster_blocks=min_cluster_blocks)
    out = kb.paged_decode_attn_shared(ctx, cache, plan, q)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), plan.info


@pytest.mark.parametrize("case", ["bf16_prefix_gqa4", "bf16_d64_gqa8_t32", "bf16_one_request", "f32_ragged", "bf16_unfused"])
@pytest.mark.parametrize("min_cluster_blocks", [1, 4])
def test_shared_decode_matches_oracle_and_plain_decode(kb, oracle, case, min_cluster_blocks):
    """Attention through the cluster plan equals the definition (the oracle's fp64 attention through the fused table)
    to the same bound as the per-request kernel, and the per-request kernel's output closely: only the order in which
    partial softmax states are merged differs."""
    _say("shared decode case", case, "min_cluster_blocks", min_cluster_blocks)
    thr = None
    if case == "bf16_prefix_gqa4":          # a common prefix (cluster of all requests) plus scattered near duplicates
        rec = wl.llama8b_bff(n_req=7, tokens=16 * 41, layers=2, kv_heads=2, prefix_tokens=16 * 9, near_pool=16)
    elif case == "bf16_d64_gqa8_t32":       # 8 query heads per KV head: two requests fill the 16 rows
        rec = wl.zipf_bff(n_req=5, tokens=32 * 9, layers=1, kv_heads=2, pool=30, t=32, d=64)
    elif case == "bf16_one_request":        # chunks of one request: blocks shared inside a request never form a cluster
        rec = wl.cff_long(tokens=16 * 300, chunk_tokens=16 * 50, layers=1, kv_heads=2)
    elif case == "f32_ragged":              # partial last blocks, mixed lengths
        rec = wl.mixed(n_req=6, min_tokens=20, max_tokens=700, chunk_tokens=256, layers=1, kv_heads=2, pool=40,
                       dtype=torch.float32)
    else:                                   # nothing fused: every block is private, the plan has no cluster
        rec = wl.llama8b_bff(n_req=4, tokens=16 * 20, layers=1, kv_heads=2, prefix_tokens=64, near_pool=8)
        thr = 1.5
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, thr=thr)
    q = wl.queries(rec, DEV)
    plain = _decode(kb, ctx, rec, cache, q)
    shared, info = _decode_shared(kb, ctx, rec, cache, q, min_cluster_blocks)
    _say("  clusters", info.clusters, "shared instances", info.shared_instances, "of", info.logical_blocks,
         "block reads", info.cluster_block_reads, "+", info.residual_block_reads)
    full_blocks = sum(int(c) // rec.t for c in rec.ctx_len) * rec.G
    assert info.logical_blocks == sum((int(c) + rec.t - 1) // rec.t for c in rec.ctx_len) * rec.G
    assert 0 <= info.shared_instances <= full_blocks
    if case == "bf16_prefix_gqa4":
        assert info.clusters >= rec.G and info.shared_instances >= rec.G * 7 * 9      # the common prefix at least
        assert info.cluster_block_reads + info.residual_block_reads < info.logical_blocks
    if case in ("bf16_unfused", "bf16_one_request"):
        assert info.clusters == 0 and info.residual_block_reads == info.logical_blocks
    worst = 0.0
    for layer in range(rec.layers):
        ref = _attn_oracle(oracle, rec, cache, q[layer], layer, rec.kv_heads)
        worst = max(worst, float(np.abs(shared[layer] - ref).max()))
    _say("  max abs err vs oracle", worst, " vs per-request kernel", float(np.abs(shared - plain).max()))
    assert worst <= 2e-2
    assert worst <= (1e-4 if rec.dtype == torch.float32 else 5e-3)
    assert np.abs(shared - plain).max() <= (1e-5 if rec.dtype == torch.float32 else 2e-3)


def test_shared_decode_rejects_bad_arguments(kb):
    rec = wl.tiny_bff()
    mat = wl.materialise(rec, DEV)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    with pytest.raises(kb.KvfuseError):       # request runs past the table
        kb.SharedDecodePlan(ctx, cache, rec.kv_heads, [rec.n - 1], [rec.t * 4], rec.q_heads)
    with pytest.raises(kb.KvfuseError):       # query heads not a multiple of KV heads
        kb.SharedDecodePlan(ctx, cache, rec.kv_heads, rec.req_start, rec.ctx_len, rec.q_heads + 1)
    with pytest.raises(kb.KvfuseError):
        kb.SharedDecodePlan(ctx, cache, rec.kv_heads, rec.req_start, rec.ctx_len, rec.q_heads, min_cluster_blocks=0)


# ------------------------------------------------------------------------------------------ chunked prefill with reuse

@pytest.mark.parametrize("case", ["d128_gqa4_last_chunk", "d64_gqa8_t32", "first_chunk_no_prefix", "unfused"])
def test_prefill_attention_with_reuse_matches_oracle(kb, oracle, case):
    """Causal attention of a ragged run of query tokens through a CFF-fused table: with reuse of fused blocks, and
    without (every logical block on its own), against the fp64 definition; the two GPU results agree closely."""
    _say("prefill case", case)
    thr = None
    if case == "d64_gqa8_t32":
        rec = wl.cff_long(tokens=32 * 120, chunk_tokens=32 * 20, layers=1, kv_heads=2, t=32, d=64)
        rec.q_heads = 8 * rec.kv_heads
        chunk_begin, q_begin, q_end = 32 * 100, 32 * 100 + 13, 32 * 100 + 13 + 70
    elif case == "first_chunk_no_prefix":
        rec = wl.cff_long(tokens=16 * 200, chunk_tokens=16 * 50, layers=1, kv_heads=2)
        chunk_begin, q_begin, q_end = 0, 0, 53
    else:
        rec = wl.cff_long(tokens=16 * 300, chunk_tokens=16 * 50, layers=2, kv_heads=2)
        chunk_begin, q_begin, q_end = 16 * 250, 16 * 250 + 37, 16 * 250 + 37 + 45
        thr = 1.5 if case == "unfused" else None
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat, thr=thr)
    assert (stats.fused > 0) == (case != "unfused")
    nq = q_end - q_begin
    gen = torch.Generator(device="cpu")
    gen.manual_seed(77)
    q = torch.randn(rec.layers, nq, rec.q_heads, rec.d, generator=gen).to(torch.bfloat16).to(DEV)
    outs, infos = [], []
    for reuse in (True, False):
        pp = kb.PrefillPlan(ctx, cache, rec.kv_heads, rec.q_heads, int(rec.req_start[0]), chunk_begin, q_begin, q_end, reuse=reuse)
        outs.append(kb.prefill_attn(ctx, cache, pp, q))
        infos.append(pp.info)
    torch.cuda.synchronize()
    _say("  blocks before the chunk: logical", infos[0].logical_blocks_before_chunk, "stored", infos[0].stored_blocks_before_chunk)
    assert infos[1].stored_blocks_before_chunk == infos[1].logical_blocks_before_chunk == rec.G * (chunk_begin // rec.t)
    assert infos[0].stored_blocks_before_chunk <= infos[0].logical_blocks_before_chunk
    if case in ("d128_gqa4_last_chunk", "d64_gqa8_t32"):
        assert infos[0].stored_blocks_before_chunk < infos[0].logical_blocks_before_chunk      # something to reuse
    worst = 0.0
    for layer in range(rec.layers):
        gs = [layer * rec.kv_heads + h for h in range(rec.kv_heads)]
        ref = oracle.causal_prefill_attention(
            q[layer].float().cpu().numpy(), np.arange(q_begin, q_end), [wl.to_numpy_pool(cache.K[g]) for g in gs],
            [wl.to_numpy_pool(cache.V[g]) for g in gs], [cache.bt[g].cpu().numpy() for g in gs],
            [cache.scale_k[g].cpu().numpy().astype(np.float64) for g in gs],
            [cache.scale_v[g].cpu().numpy().astype(np.float64) for g in gs], int(rec.req_start[0]), rec.t, rec.d)
        for o in outs:
            worst = max(worst, float(np.abs(o[layer].cpu().numpy() - ref).max()))
    diff = float((outs[0] - outs[1]).abs().max())
    _say("  max abs err vs oracle", worst, " reuse vs no reuse", diff)
    assert worst <= 2e-2 and worst <= 5e-3 and diff <= 1e-4


def test_prefill_rejects_bad_arguments(kb):
    rec = wl.cff_long(tokens=16 * 64, chunk_tokens=16 * 16, layers=1, kv_heads=2)
    mat = wl.materialise(rec, DEV)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    for args in ((0, 8, 8, 40), (0, 16, 8, 40), (0, 16, 40, 30), (0, 16 * 32, 16 * 32, 16 * 64 + 1), (-1, 0, 0, 8)):
        with pytest.raises(kb.KvfuseError):
            kb.PrefillPlan(ctx, cache, rec.kv_heads, rec.q_heads, *args)
    with pytest.raises(kb.KvfuseError):
        kb.PrefillPlan(ctx, cache, rec.kv_heads, rec.q_heads + 1, 0, 0, 0, 8)


# ------------------------------------------------------------------------------------------ threshold control

@pytest.mark.parametrize("kind", ["bf16_fused", "f32_tiny"])
def test_pair_cosines_and_moments_match_oracle(kb, kind):
    """Sampled pair cosines through the (fused) table and their per-group moments against the definition."""
    import oracle as oracle_pkg
    from oracle import threshold as th
    _say("pair cosines", kind)
    rec = _small_bf16(n_req=5, tokens=640, kv_heads=2) if kind == "bf16_fused" else wl.tiny_bff()
    mat = wl.materialise(rec, DEV, phys_perm=True)
    cache, plan, stats, ctx = gu.gpu_fuse(rec, mat)
    assert stats.fused > 0
    rng = np.random.default_rng(17)
    n_pairs = 777
    pairs_h = rng.integers(0, rec.n, size=(n_pairs, 2)).astype(np.int32)
    pairs_h[0] = (3, 3)                                    # a block with itself
    pairs = torch.tensor(pairs_h, device=DEV)
    cos = kb.pair_cosines(ctx, cache, pairs)
    mom = kb.cosine_moments(ctx, cos)
    torch.cuda.synchronize()
    cos_h, mom_h = cos.cpu().numpy(), mom.cpu().numpy()
    for g in range(rec.G):
        Kf = oracle_pkg.pool_to_f64(wl.to_numpy_pool(cache.K[g]))
        want = th.pair_cosines(Kf.reshape(Kf.shape[0], -1), cache.bt[g].cpu().numpy(), pairs_h)
        np.testing.assert_allclose(cos_h[g], want, rtol=1e-12, atol=1e-15)
        assert cos_h[g][0] == pytest.approx(1.0, abs=1e-14)
        mu, var = th.moments(want)
        assert mom_h[g][0] == pytest.approx(mu, rel=1e-11, abs=1e-14) and mom_h[g][1] == pytest.approx(var, rel=1e-10)
    # the library's rate on these moments equals the oracle's
    mu, var = float(mom_h[0][0]), float(mom_h[0][1])
    assert kb.exceedance_rate(1e6, mu, math.sqrt(var), rec.thr) == pytest.approx(th.exceedance_rate(1e6, mu, math.sqrt(var), rec.thr), rel=1e-12, abs=1e-300)


@pytest.mark.parametrize("screen", ["full_product", "both_screens"])
def test_group_mask_skips_groups_and_leaves_the_rest_unchanged(kb, oracle, screen):
    """A switched-off group comes out of the tree untouched; the other groups are bit-identical to an unmasked run (which
    uses the full product, also when the masked run goes through the two screens)."""
    _say("group mask", screen)
    rec = _small_bf16(n_req=6, tokens=800, kv_heads=4)
    mat_a = wl.materialise(rec, DEV, phys_perm=True)
    cache_a, plan_a, stats_a, ctx = gu.gpu_fuse(rec, mat_a)
    mat_b = wl.materialise(rec, DEV, phys_perm=True)
    K0, V0, bt0 = mat_b["K"].clone(), mat_b["V"].clone(), mat_b["bt"].clone()
    cache_b = kb.Cache(mat_b["K"], mat_b["V"], mat_b["bt"], rec.t, rec.d)
    plan_b = kb.Plan(ctx, cache_b, kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.group_size), 16)
    if screen == "both_screens":
        kb.set_screen_fp8(ctx, plan_b)
        kb.set_screen_prefix(ctx, plan_b, 128)
    mask = torch.tensor([1, 0, 1, 0], dtype=torch.uint8, device=DEV)
    kb.set_group_mask(ctx, plan_b, mask)
    stats_b = kb.fuse_tree(ctx, plan_b, rec.thr, want_stats=True)
    torch.cuda.synchronize()
    for g in range(rec.G):
        if int(mask[g]):
            assert torch.equal(cache_b.bt[g], cache_a.bt[g]) and torch.equal(cache_b.K[g], cache_a.K[g])
            assert torch.equal(cache_b.V[g], cache_a.V[g]) and torch.equal(cache_b.scale_k[g], cache_a.scale_k[g])
        else:
            assert torch.equal(cache_b.bt[g], bt0[g]) and torch.equal(cache_b.K[g], K0[g]) and torch.equal(cache_b.V[g], V0[g])
            assert bool((cache_b.scale_k[g] == 1).all()) and bool((cache_b.refcount[g][bt0[g].long()] == 1).all())
    assert 0 < stats_b.fused < stats_a.fused and stats_b.sim_flops < stats_a.sim_flops
    # and back to all groups
    kb.set_group_mask(ctx, plan_b, None)
    cache_b.K.copy_(K0); cache_b.V.copy_(V0); cache_b.bt.copy_(bt0)
    stats_c = kb.fuse_tree(ctx, plan_b, rec.thr, want_stats=True)
    assert stats_c.fused == stats_a.fused and torch.equal(cache_b.bt, cache_a.bt)


# ------------------------------------------------------------------------------------------ machine probes

def test_machine_probes_run_and_copy_is_exact():
    """The probe library (its own .so and header, used by bench.py only): every probe runs, the copy is exact, the
    read-two-write-one pattern touches what it says, bad arguments come back as errors."""
    from paper_2601_03067_amd import probe as kp
    _say("machine probes")
    a = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    b = torch.zeros_like(a)
    gbps = kp.copy(a, b, repeats=2)
    assert gbps > 0 and torch.equal(a, b)
    rnd = kp.mfma_bf16(True, DEV)
    const = kp.mfma_bf16(False, DEV)
    _say("  mfma bf16 TFLOP/s: random operands", round(rnd), "constant operands", round(const), "copy GB/s (small)", round(gbps))
    assert 50 < rnd < 2600 and 50 < const < 2600      # below the nominal dense peak of 2500 plus timing slack
    rnd8, const8 = kp.mfma_fp8(True, DEV), kp.mfma_fp8(False, DEV)
    _say("  mfma fp8 TFLOP/s: random operands", round(rnd8), "constant operands", round(const8))
    assert 50 < rnd8 < 5200 and 50 < const8 < 5200    # nominal dense fp8 peak 5000
    data = torch.randn(4 << 20, device=DEV).to(torch.bfloat16)          # 8 MiB of cache-like values
    loop = kp.tile_loop_bf16(data, True)
    loop0 = kp.tile_loop_bf16(data, False)
    _say("  stripped tile loop TFLOP/s: with loads", round(loop), "without", round(loop0))
    assert 50 < loop < 2600 and 50 < loop0 < 2600
    with pytest.raises(kp.ProbeError):
        kp.tile_loop_bf16(data[:1000], True)                 # less than 4 MiB
    # the merge access pattern: item i of a 256-block stripe xors block i + 128 into block i (i < 32) and nothing else
    # moves; the probe runs its kernel an even number of times here (warm-up + 1), which must restore the buffer
    blk = 4096
    buf = torch.randint(0, 2 ** 31 - 1, (3 * 256 + 7, blk // 4), dtype=torch.int32, device=DEV)   # three stripes and a bit
    orig = buf.clone()
    rate = kp.read2_write1(buf, blk, repeats=1)
    torch.cuda.synchronize()
    assert rate > 0 and torch.equal(buf, orig)
    kp.read2_write1(buf, blk, repeats=2)               # three applications = one
    torch.cuda.synchronize()
    want = orig.clone()
    for s0 in range(0, 3 * 256, 256):
        want[s0:s0 + 32] ^= want[s0 + 128:s0 + 160]
    assert torch.equal(buf, want)
    with pytest.raises(kp.ProbeError):
        kp.read2_write1(buf[:100], blk)                # smaller than one stripe
    assert kp.lib.kvfuse_probe_copy(None, None, None, 0, 1, None) == 1      # KVFUSE_PROBE_EINVAL
