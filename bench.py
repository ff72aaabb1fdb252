#!/usr/bin/env python3
"""Benchmark of the Fast Fusion hot path on ONE MI355X.

A step = one pass of the whole hot path over one batch of synthetic input that is already resident in HBM:
block norms -> per tree height (similarity, assignment, merge) -> block-table rewrite -> one decode-attention
step of every request over every layer through the fused table.  Fusion rewrites the pool in place, so the pool
and table are restored from a device snapshot between steps, outside the timed region.

Prints ONE JSON line.  `value` = logical KV blocks (per layer and KV head) pushed through the whole path per
second.  `roofline` describes the dominant kernel, the MFMA similarity GEMM: algorithmic flops (2 m_l m_r r per
tree node with the actual set sizes) over its HIP-event time on the launch stream.  `cpu_baseline` times the CPU
oracle on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def make_recipe(wl, name):
    if name == "llama8b_bff":
        return wl.llama8b_bff()
    if name == "cff_long":
        return wl.cff_long()
    if name == "tiny_bff":
        return wl.tiny_bff()
    if name == "llama8b_bff_prefix75":       # same shape, three quarters of every request is the common prefix
        return wl.llama8b_bff(prefix_tokens=1536)
    if name == "zipf_bff_slab":              # config 4's shape, a slab of 4 of its 80 layers (the whole does not fit HBM un-fused)
        return wl.zipf_bff(layers=4)
    if name == "mixed_slab":                 # config 5's shape, one of its 32 layers (292 GB un-fused as a whole)
        return wl.mixed(layers=1)
    if name == "llama8b_bff_small":          # quick functional check, not a benchmark configuration
        return wl.llama8b_bff(n_req=16, layers=4)
    raise SystemExit(f"unknown workload {name}")


# The two configurations whose un-fused cache exceeds one GPU's HBM: name -> (full recipe, layers per slab, thresholds).
# Layers are independent in every step of the path (method section: one table per layer), so such a configuration is
# processed in slabs of layers that are generated, fused and decoded one after the other in the same buffers, and its
# totals are sums over the slabs.
WHOLE_CONFIGS = {
    "zipf_bff": (lambda wl: wl.zipf_bff(), 4, (0.85, 0.9, 0.95)),        # config 4: 80 layers, 344 GB un-fused
    "mixed": (lambda wl: wl.mixed(), 4, (0.9,)),                          # config 5: 32 layers, 292 GB un-fused
}


def run_whole_config(args, torch, kb, wl):
    """Config 4 or 5 as a whole: every layer slab, every threshold of the configuration, decode attention for every
    request on every layer.  One JSON line; `value` = all logical blocks of all layers over the summed step times."""
    make, slab_layers, thresholds = WHOLE_CONFIGS[args.workload]
    rec = make(wl)
    if args.thr is not None:
        thresholds = (args.thr,)
    if args.slab_layers:
        slab_layers = args.slab_layers
    dev = "cuda:0"
    H = rec.kv_heads
    if rec.layers % slab_layers:
        raise SystemExit(f"--slab-layers must divide the {rec.layers} layers of {rec.name}")
    n_slabs = rec.layers // slab_layers
    if args.max_slabs:
        n_slabs = min(n_slabs, args.max_slabs)
    Gs = slab_layers * H
    elem = 2 if rec.dtype == torch.bfloat16 else 4
    K = torch.empty(Gs, rec.n, rec.r, device=dev, dtype=rec.dtype)
    V = torch.empty_like(K)
    bt = torch.empty(Gs, rec.n, device=dev, dtype=torch.int32)
    K0, V0, bt0 = torch.empty_like(K), torch.empty_like(V), torch.empty_like(bt)
    ctx = kb.Context(dev)
    cache = kb.Cache(K, V, bt, rec.t, rec.d)
    spec = kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.group_size)
    plan = kb.Plan(ctx, cache, spec, args.cand_cap)
    if args.screen_fp8:
        kb.set_screen_fp8(ctx, plan, centre=args.centre)
    if args.screen_prefix:
        kb.set_screen_prefix(ctx, plan, args.screen_prefix)
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=dev)
    cl = torch.tensor(rec.ctx_len, dtype=torch.int32, device=dev)
    max_blocks = int(((rec.ctx_len + rec.t - 1) // rec.t).max())
    ws = torch.empty(kb.decode_workspace_bytes(slab_layers, rec.B, rec.q_heads, H, rec.d, max_blocks), device=dev, dtype=torch.uint8)
    out = torch.empty(slab_layers, rec.B, rec.q_heads, rec.d, device=dev, dtype=torch.float32)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    per_thr = {}
    t_gen = 0.0
    for si in range(n_slabs):
        layers = list(range(si * slab_layers, min(rec.layers, (si + 1) * slab_layers)))
        t0 = time.perf_counter()
        for li, layer in enumerate(layers):
            m = wl.materialise(rec, dev, groups=range(layer * H, (layer + 1) * H))
            K0[li * H:(li + 1) * H].copy_(m["K"]); V0[li * H:(li + 1) * H].copy_(m["V"]); bt0[li * H:(li + 1) * H].copy_(m["bt"])
            del m
        q = wl.queries(rec, dev, layers=layers)
        torch.cuda.synchronize()
        t_gen += time.perf_counter() - t0
        for thr in thresholds:
            acc = per_thr.setdefault(thr, {"ms": [], "stage": {}, "fused": 0, "physical": 0, "logical": 0, "flops": 0.0,
                                           "refined": 0, "overflow": 0, "near": 0, "targets": 0})
            reps = args.steps + (args.warmup if si == 0 else 0)
            for rep in range(reps):
                K.copy_(K0); V.copy_(V0); bt.copy_(bt0)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                ev[0].record()
                st = kb.fuse_tree(ctx, plan, thr, want_stats=True, want_timing=True)
                ev[1].record()
                kb.paged_decode_attn(ctx, cache, H, q, rs, cl, max_blocks, workspace=ws, out=out)
                ev[2].record()
                torch.cuda.synchronize()
                wall = (time.perf_counter() - t1) * 1e3
                if si == 0 and rep < args.warmup:
                    continue
                acc["ms"].append(wall / 1.0)
                for k2, v2 in (("norms", st.ms_norms), ("similarity", st.ms_similarity), ("assign", st.ms_assign),
                               ("merge", st.ms_merge), ("rewrite", st.ms_rewrite), ("decode", ev[1].elapsed_time(ev[2]))):
                    acc["stage"][k2] = acc["stage"].get(k2, 0.0) + v2 / args.steps
                if rep == reps - 1:
                    acc["fused"] += st.fused; acc["physical"] += st.physical_blocks; acc["logical"] += st.logical_blocks
                    acc["flops"] += st.sim_flops; acc["refined"] += st.refined; acc["overflow"] += st.cand_overflow
                    acc["near"] += st.near_threshold; acc["targets"] += st.merge_targets
        print(f"bench.py: slab {si + 1}/{n_slabs} (layers {layers[0]}..{layers[-1]}) done, "
              + ", ".join(f"thr {t}: {per_thr[t]['ms'][-1]:.1f} ms" for t in thresholds), file=sys.stderr, flush=True)
    main_thr = rec.thr if rec.thr in per_thr else thresholds[0]
    a = per_thr[main_thr]
    slab_ms = [sum(a["ms"][i * args.steps:(i + 1) * args.steps]) / args.steps for i in range(n_slabs)]
    total_ms = sum(slab_ms)
    blocks = a["logical"]
    peak = 2500.0 if rec.dtype == torch.bfloat16 else 157.3
    sim_tflops = a["flops"] / (a["stage"]["similarity"] * 1e-3) / 1e12
    phys_bytes = a["physical"] * rec.r * elem * 2
    line = {
        "metric": "KV blocks fused/sec (+ % MFMA peak); fused-table decode attn HBM GB/s",
        "value": blocks / (total_ms * 1e-3), "unit": "blocks/s",
        "value_is": "logical KV blocks of ALL layers through norms, the whole fusion tree and one decode-attention step, over the "
                    "summed step times of the layer slabs (the un-fused cache exceeds one GPU's HBM; layers are independent, "
                    "so the configuration runs slab after slab in the same buffers and totals are sums over slabs)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": total_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if rec.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": f"{rec.name} (whole configuration): {rec.layers} layers x {H} KV heads in {n_slabs} slabs of "
                               f"{slab_layers} layers, d {rec.d}, block {rec.t}, {rec.B} requests, {rec.n} logical blocks per group, "
                               f"thr {main_thr}; decode attention for every request on every layer",
                   "groups": n_slabs * Gs, "logical_blocks": blocks, "physical_blocks_after": a["physical"],
                   "compression_ratio": blocks / a["physical"] if a["physical"] else 0.0, "fused": a["fused"],
                   "near_threshold": a["near"], "refined_fp64": a["refined"], "cand_overflow": a["overflow"],
                   "slabs": n_slabs, "slab_layers": slab_layers,
                   "screen": (("centred fp8 copies" if args.centre else "fp8 copies") if args.screen_fp8 else "full product") + (f", prefix of {args.screen_prefix}" if args.screen_prefix else ""),
                   "unfused_cache_GB": rec.layers * H * rec.n * rec.r * elem * 2 / 1e9},
        "stages_ms": a["stage"],
        "per_slab_ms": {"min": min(slab_ms), "median": sorted(slab_ms)[len(slab_ms) // 2], "max": max(slab_ms), "all": slab_ms},
        "thresholds": {str(t): {"ms_total": sum(per_thr[t]["ms"]) / args.steps, "compression_ratio": per_thr[t]["logical"] / max(per_thr[t]["physical"], 1),
                                "fused": per_thr[t]["fused"], "refined_fp64": per_thr[t]["refined"], "stages_ms": per_thr[t]["stage"]}
                       for t in thresholds},
        "decode": {"ms": a["stage"]["decode"], "physical_GBps": phys_bytes / (a["stage"]["decode"] * 1e-3) / 1e9,
                   "frac_of_hbm_peak_physical": phys_bytes / (a["stage"]["decode"] * 1e-3) / 1e9 / 8000.0},
        "merge": {"ms": a["stage"]["merge"],
                  "GBps": (2 * a["targets"] + a["fused"]) * rec.r * elem * 2 / (a["stage"]["merge"] * 1e-3) / 1e9},
        "roofline": {"kernel": "similarity_ring_kernel", "bound": "mfma", "achieved": sim_tflops, "peak": peak, "unit": "TFLOP/s",
                     "frac": sim_tflops / peak, "traffic": None, "flops_total": a["flops"], "ms_total": a["stage"]["similarity"]},
        "generation_s": t_gen,
    }
    print(json.dumps(line))


def cpu_baseline(wl, reduced=False):
    """Time the oracle (as it stands) on the host cores over a bounded sample of the workload the GPU is timed on:
    one group per core (at least 8 groups) of the llama8b_bff recipe at its full per-group shape, 64 requests x 128
    blocks, through the same unit of work as `value`: norms + Algorithm 1's whole tree, then one decode-attention
    step of every request through the fused table.  ``reduced`` (a labelled fallback for quick runs) halves the
    request count."""
    import numpy as np
    import oracle
    import torch
    cores = min(16, os.cpu_count() or 1)
    groups = max(8, cores)
    n_req = 32 if reduced else 64
    rec = wl.llama8b_bff(n_req=n_req, layers=1, kv_heads=groups)
    dev = "cuda:0" if torch.cuda.is_available() else "cpu"
    mat = wl.materialise(rec, dev)
    Ks = [wl.to_numpy_pool(mat["K"][g]) for g in range(rec.G)]
    Vs = [wl.to_numpy_pool(mat["V"][g]) for g in range(rec.G)]
    bts = [mat["bt"][g].cpu().numpy() for g in range(rec.G)]
    q = wl.queries(rec, dev)[0].float().cpu().numpy()
    del mat
    oracle.build()
    t0 = time.perf_counter()
    res = oracle.fuse_groups(Ks, Vs, bts, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr, threads=cores)
    t_fuse = time.perf_counter() - t0
    # decode: the groups are the KV heads of one layer; requests are shared out over the same threads
    from concurrent.futures import ThreadPoolExecutor

    def dec(b):
        return oracle.paged_decode_attention(q[b: b + 1], [r.kpool for r in res], [r.vpool for r in res], [r.bt for r in res],
                                             [r.scale_k for r in res], [r.scale_v for r in res], rec.req_start[b: b + 1],
                                             rec.ctx_len[b: b + 1], rec.t, rec.d)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        outs = list(ex.map(dec, range(rec.B)))
    t_dec = time.perf_counter() - t0
    assert np.isfinite(np.concatenate(outs)).all()
    dt = t_fuse + t_dec
    blocks = rec.G * rec.n
    model = "unknown"
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"value": blocks / dt, "unit": "blocks/s", "cores": cores, "kind": "oracle", "cpu_model": model,
            "blocks_per_s_per_core": blocks / dt / cores,
            "fusion_s": t_fuse, "decode_s": t_dec,
            "sample": f"{rec.G} groups (one layer of {rec.G} KV heads) x {n_req} requests x 128 blocks of the llama8b_bff recipe"
                      f"{' -- REDUCED sample, half the requests of the timed shape' if reduced else ', the per-group shape the GPU is timed on'}: "
                      f"norms + fusion ({t_fuse:.1f} s wall, one group per thread) + decode attention of all {rec.B} requests "
                      f"({t_dec:.1f} s), CR {sum(len(r.bt) for r in res) / sum(r.n_physical for r in res):.3f}; same unit as "
                      f"`value`: logical blocks through norms, fusion and decode per second"}


class PowerSampler:
    """Socket power from the amdgpu hwmon node (power1_input / power1_average, microwatts), read every few
    milliseconds by a host thread while a GPU loop runs.  Readings only; nothing on the GPU is touched."""

    def __init__(self):
        import glob
        self.files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                            glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))[:1]
        caps = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap"))
        self.cap_W = None
        try:
            self.cap_W = float(open(caps[0]).read()) / 1e6 if caps else None
        except (OSError, ValueError):
            pass

    def measure(self, fn, seconds, sync):
        """Run fn() back to back for about `seconds`; return (ms per call, mean W, max W) over the later two thirds."""
        import threading
        samples, stop = [], [False]

        def loop():
            while not stop[0]:
                try:
                    samples.append(float(open(self.files[0]).read()) / 1e6)
                except (OSError, ValueError, IndexError):
                    pass
                time.sleep(0.004)
        th = threading.Thread(target=loop)
        th.start()
        sync()
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < seconds:
            fn()
            sync()
            n += 1
        dt = time.perf_counter() - t0
        stop[0] = True
        th.join()
        tail = samples[len(samples) // 3:]
        return dt / n * 1e3, (sum(tail) / len(tail) if tail else None), (max(tail) if tail else None)


def power_report(kb, kp, ctx, cache, plan, rec, restore, torch, decode_step=None):
    """Socket power while the similarity stage runs on full sets, next to the machine probes and an HBM-bound kernel:
    shows which limit the dominant kernel runs at (the board's power cap is read from the same hwmon node)."""
    ps = PowerSampler()
    if not ps.files:
        return {"error": "no hwmon power node readable"}
    dev = cache.K.device
    sync = lambda: torch.cuda.synchronize(dev)
    restore()
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)

    def sim_tree():        # nothing fuses above 1: every similarity launch of the tree on full sets
        kb.leaf_sets(ctx, plan)
        for h in range(plan.n_heights):
            kb.similarity(ctx, plan, h, 1.5, 1e-3, None)
            kb.assign(ctx, plan, h, 1.5, 1e-3)
    out = {"cap_W": ps.cap_W, "sensor": ps.files[0]}
    ms, mean, mx = ps.measure(lambda: time.sleep(0.05), 1.0, sync)
    out["idle"] = {"mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(sim_tree, 2.5, sync)
    out["similarity_all_heights_full_sets"] = {"ms": ms, "mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(lambda: kp.mfma_bf16(True, dev), 2.0, sync)
    out["mfma_probe_random_operands"] = {"mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(lambda: kp.mfma_bf16(False, dev), 2.0, sync)
    out["mfma_probe_constant_operands"] = {"mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(lambda: kp.mfma_fp8(True, dev), 2.0, sync)
    out["mfma_fp8_probe_random_operands"] = {"mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(lambda: kp.mfma_fp8(False, dev), 2.0, sync)
    out["mfma_fp8_probe_constant_operands"] = {"mean_W": mean, "max_W": mx}
    ms, mean, mx = ps.measure(lambda: kb.block_norms(ctx, cache), 1.5, sync)
    out["block_norms_hbm_stream"] = {"ms": ms, "mean_W": mean, "max_W": mx}
    if decode_step is not None:         # decode attention over the un-fused cache: the other HBM stream of a step
        cache.identity_scales()
        ms, mean, mx = ps.measure(decode_step, 1.5, sync)
        out["decode_unfused_hbm_stream"] = {"ms": ms, "mean_W": mean, "max_W": mx}
    cache.K.zero_()
    kb.block_norms(ctx, cache)
    ms, mean, mx = ps.measure(sim_tree, 2.5, sync)
    out["similarity_all_heights_full_sets_zero_pool"] = {"ms": ms, "mean_W": mean, "max_W": mx}
    restore()
    return out


def similarity_tile_model(ml, mr, big):
    """What the similarity kernel's tiling issues for nodes with ``ml`` left and ``mr`` right blocks (integer arrays
    of one shape): rows and columns of MFMA work per node after the skipped bands (sum over its tiles; work =
    rows x cols x 2 r flops is exact because the bands of a tile are whole in both directions), and the rows loaded
    into LDS (every tile of BM x BN loads BM + BN block rows, ragged or not).  Bookkeeping for benchmarks: mirrors
    the launch geometry of csrc/similarity.hip, computes nothing of the method."""
    import numpy as np
    ml = np.asarray(ml, np.int64)
    mr = np.asarray(mr, np.int64)
    bm = bn = 256 if big else 128
    row_band, col_band = (128, 64) if big else (64, 64)
    n_rt = -(-ml // bm)
    n_cp = -(-mr // bn)
    full_r, tail_r = ml // bm, ml % bm
    full_c, tail_c = mr // bn, mr % bn
    rows = full_r * bm + -(-tail_r // row_band) * row_band
    cols = full_c * bn + -(-tail_c // col_band) * col_band
    rows = np.where(mr > 0, rows, 0)
    cols = np.where(ml > 0, cols, 0)
    loaded_rows = n_rt * n_cp * (bm + bn)
    return rows, cols, loaded_rows


def per_height_table(kb, ctx, cache, plan, rec, restore, thr):
    """One extra fusion pass taken height by height (similarity, assignment, merge as separate calls with HIP events
    around the similarity launch): per tree height the node count, the mean set sizes, the valid flops
    2 m_l m_r r, the MFMA work the tiling issues for those sizes (whole 32 x 32 MFMA tiles that are not skipped),
    the bytes the tiling loads into LDS, and the time.  Used for profiles/: where the similarity stage loses
    against its own full-tile rate is read off this table."""
    import numpy as np
    import torch
    dev = cache.K.device
    restore()
    kb.block_norms(ctx, cache)
    kb.leaf_sets(ctx, plan)
    # bytes per element of what the similarity kernel reads: the pool, or its one-byte copy under the fp8 screen
    elem = 1 if getattr(plan, "k8", None) is not None else (2 if rec.dtype == torch.bfloat16 else 4)
    rows = []
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for h in range(plan.n_heights):
        v = plan.view(h)
        torch.cuda.synchronize()
        ev[0].record()
        kb.similarity(ctx, plan, h, thr, 1e-3, None)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1])
        cnt = kb.device_array(v.set_cnt, rec.G * v.n_slots, np.int32, dev).reshape(rec.G, v.n_slots).astype(np.int64)
        ml = cnt[:, kb.device_array(v.l_slot, v.n_nodes, np.int32, dev)]
        mr = cnt[:, kb.device_array(v.r_slot, v.n_nodes, np.int32, dev)]
        lcap = kb.device_array(v.l_cap, v.n_nodes, np.int32, dev).astype(np.int64)
        rcap = kb.device_array(v.r_cap, v.n_nodes, np.int32, dev).astype(np.int64)
        wsum = float((lcap * rcap).sum())
        big = wsum > 0 and float((lcap * rcap * np.minimum(lcap, rcap)).sum()) / wsum >= 256.0     # the plan's rule
        mma_rows, mma_cols, lds_bytes = similarity_tile_model(ml, mr, big)
        valid = float((2 * ml * mr).sum()) * rec.r
        tile = float((2 * mma_rows * mma_cols).sum()) * rec.r
        kb.assign(ctx, plan, h, thr, 1e-3)
        kb.merge(ctx, plan, h)
        rows.append({"height": h + 1, "nodes_per_group": int(v.n_nodes), "tile": "256x256" if big else "128x128",
                     "mean_m_l": float(ml.mean()), "mean_m_r": float(mr.mean()), "valid_TFLOP": valid / 1e12,
                     "mfma_TFLOP": tile / 1e12, "valid_over_mfma": valid / tile if tile else 0.0,
                     "lds_load_GB": float(lds_bytes.sum()) * rec.r * elem / 1e9,
                     "compulsory_GB": float((ml + mr).sum()) * rec.r * elem / 1e9, "ms": ms,
                     "valid_TFLOPs": valid / ms / 1e9 if ms else 0.0, "mfma_TFLOPs": tile / ms / 1e9 if ms else 0.0})
    torch.cuda.synchronize()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama8b_bff")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-reduced", action="store_true",
                    help="time the oracle on half the requests per group (quick runs; labelled as reduced in the output)")
    ap.add_argument("--cand-cap", type=int, default=64)
    ap.add_argument("--thr", type=float, default=None, help="override the workload's similarity threshold")
    ap.add_argument("--assign-rule", choices=["argmax", "first_row"], default="argmax",
                    help="reading of Algorithm 1's threshold line: most similar row, or first row above the threshold")
    ap.add_argument("--shortest-first", action="store_true",
                    help="build the tree over the requests in ascending number of blocks (remark on the order of requests)")
    ap.add_argument("--slab-layers", type=int, default=0, help="layers per slab of a whole-configuration run (zipf_bff, mixed)")
    ap.add_argument("--max-slabs", type=int, default=0, help="stop a whole-configuration run after this many slabs (quick checks)")
    ap.add_argument("--screen-prefix", type=int, default=0,
                    help="elements of every key block the similarity screen multiplies in the TIMED steps (0 = whole blocks, the "
                         "default; the opt-in prefix screen is measured outside the timed steps either way)")
    ap.add_argument("--screen-fp8", action="store_true",
                    help="run the timed steps with the fp8 screen (similarity over one-byte copies of the key blocks + error bound)")
    ap.add_argument("--centre", action="store_true",
                    help="with --screen-fp8: take each group's common key direction out of the one-byte copies first")
    ap.add_argument("--common-direction", action="store_true",
                    help="after the timed steps, also run the full product and the fp8 screen (plain and centred copies) on keys "
                         "that share a direction (field fp8_screen.keys_with_a_common_direction; a few seconds)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--per-height", action="store_true",
                    help="after the timed steps, run one more fusion height by height and add a per-height table of the "
                         "similarity stage (set sizes, valid and issued MFMA work, bytes loaded, time) to the output")
    ap.add_argument("--power", action="store_true",
                    help="after the timed steps, sample the socket power (hwmon) while the similarity stage, the MFMA probes and "
                         "the norm pass run, and add the readings and the board's power cap to the output")
    ap.add_argument("--calib-copy-gib", type=float, default=0.0,
                    help="also run a plain device copy of this many GiB (3 times) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path (groups would shard with no "
                         "exchange); run with --gpus 1")

    import torch
    from paper_2601_03067_amd import binding as kb
    from paper_2601_03067_amd import probe as kp
    from paper_2601_03067_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload in WHOLE_CONFIGS:
        run_whole_config(args, torch, kb, wl)
        return
    dev = "cuda:0"
    rec = make_recipe(wl, args.workload)
    if args.thr is not None:
        rec.thr = args.thr
    t_gen = time.perf_counter()
    mat = wl.materialise(rec, dev)
    q = wl.queries(rec, dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    K0, V0, bt0 = mat["K"].clone(), mat["V"].clone(), mat["bt"].clone()

    ctx = kb.Context(dev)
    cache = kb.Cache(mat["K"], mat["V"], mat["bt"], rec.t, rec.d)
    spec = kb.tree_spec(rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.group_size)
    if args.shortest_first:
        spec, _ = kb.tree_spec_shortest_first(spec)
    plan = kb.Plan(ctx, cache, spec, args.cand_cap)
    rule = {"argmax": kb.RULE_ARGMAX, "first_row": kb.RULE_FIRST_ROW}[args.assign_rule]
    kb.set_assign_rule(ctx, plan, rule)
    if args.screen_fp8:
        kb.set_screen_fp8(ctx, plan, centre=args.centre)
    if args.screen_prefix:
        kb.set_screen_prefix(ctx, plan, args.screen_prefix)
    rs = torch.tensor(rec.req_start, dtype=torch.int32, device=dev)
    cl = torch.tensor(rec.ctx_len, dtype=torch.int32, device=dev)
    max_blocks = int(((rec.ctx_len + rec.t - 1) // rec.t).max())
    ws = torch.empty(kb.decode_workspace_bytes(rec.layers, rec.B, rec.q_heads, rec.kv_heads, rec.d, max_blocks),
                     device=dev, dtype=torch.uint8)
    out = torch.empty(rec.layers, rec.B, rec.q_heads, rec.d, device=dev, dtype=torch.float32)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def restore():
        cache.K.copy_(K0)
        cache.V.copy_(V0)
        cache.bt.copy_(bt0)

    def step():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record()
        st = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True, want_timing=True)
        ev[1].record()
        kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, max_blocks, workspace=ws, out=out)
        ev[2].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return wall, st, ev[1].elapsed_time(ev[2])

    if args.calib_copy_gib > 0:
        nelem = int(args.calib_copy_gib * (1 << 30)) // 4
        src = torch.ones(nelem, device=dev, dtype=torch.int32)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.bitwise_not(src, out=dst)     # one elementwise kernel: reads nelem * 4 bytes, writes nelem * 4 bytes
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        restore()
        step()
    walls, sims, decs, stats = [], [], [], None
    stage = {"norms": 0.0, "similarity": 0.0, "assign": 0.0, "merge": 0.0, "rewrite": 0.0, "decode": 0.0}
    for _ in range(args.steps):
        restore()
        wall, st, dec = step()
        walls.append(wall)
        stats = st
        stage["norms"] += st.ms_norms; stage["similarity"] += st.ms_similarity; stage["assign"] += st.ms_assign
        stage["merge"] += st.ms_merge; stage["rewrite"] += st.ms_rewrite; stage["decode"] += dec
    # shared-block decode attention (the first "next" row): same outputs, blocks common to several requests read
    # once per tile of requests.  Measured on the table the last step left, outside the timed steps.
    t_plan = time.perf_counter()
    splan = kb.SharedDecodePlan(ctx, cache, rec.kv_heads, rec.req_start, rec.ctx_len, rec.q_heads, min_cluster_blocks=4)
    t_plan = time.perf_counter() - t_plan
    out_sh = torch.empty_like(out)
    kb.paged_decode_attn_shared(ctx, cache, splan, q, out=out_sh)
    sev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    sev[0].record()
    for _ in range(3):
        kb.paged_decode_attn_shared(ctx, cache, splan, q, out=out_sh)
    sev[1].record()
    torch.cuda.synchronize()
    ms_shared = sev[0].elapsed_time(sev[1]) / 3
    shared_diff = float((out_sh - out).abs().max())
    si = splan.info

    # chunked-prefill attention with reuse on fused blocks (a "next" row; one-request workloads only): the last chunk's
    # queries over the fused context, 4 layers, with the reuse and with every logical block on its own
    prefill = None
    if rec.B == 1 and rec.dtype == torch.bfloat16:
        chunk_tokens = int(rec.leaf_count[-1]) * rec.t
        total = int(rec.ctx_len[0])
        cb = (total - 1) // chunk_tokens * chunk_tokens
        pl_layers = min(4, rec.layers)
        gen = torch.Generator(device="cpu")
        gen.manual_seed(wl.MASTER_SEED + 7)
        qp = torch.randn(pl_layers, total - cb, rec.q_heads, rec.d, generator=gen).to(rec.dtype).to(dev)
        outp = torch.empty(pl_layers, total - cb, rec.q_heads, rec.d, device=dev, dtype=torch.float32)
        prefill = {"layers": pl_layers, "query_tokens": total - cb, "context_tokens": total}
        ref_out = None
        for reuse in (True, False):
            pp = kb.PrefillPlan(ctx, cache, rec.kv_heads, rec.q_heads, int(rec.req_start[0]), cb, cb, total, n_layers=pl_layers,
                                reuse=reuse)
            kb.prefill_attn(ctx, cache, pp, qp, out=outp)
            torch.cuda.synchronize()
            sev[0].record()
            for _ in range(2):
                kb.prefill_attn(ctx, cache, pp, qp, out=outp)
            sev[1].record()
            torch.cuda.synchronize()
            ms_p = sev[0].elapsed_time(sev[1]) / 2
            # algorithmic flops: every query row against every logical token it sees, Q.K and P.V
            seen = sum(range(cb + 1, total + 1))
            flops = 4.0 * rec.d * seen * rec.q_heads * pl_layers
            key = "reuse" if reuse else "no_reuse"
            prefill[key] = {"ms": ms_p, "TFLOPs_algorithmic": flops / (ms_p * 1e-3) / 1e12,
                            "stored_blocks_before_chunk": pp.info.stored_blocks_before_chunk,
                            "logical_blocks_before_chunk": pp.info.logical_blocks_before_chunk}
            if ref_out is None:
                ref_out = outp.clone()
            else:
                prefill["max_abs_diff_reuse_vs_no_reuse"] = float((outp - ref_out).abs().max())
        prefill["speedup_from_reuse"] = prefill["no_reuse"]["ms"] / prefill["reuse"]["ms"]

    # threshold-control statistics (another "next" row): key cosines of sampled logical pairs on the unfused cache,
    # their moments, and the analysis section's Gaussian exceedance rate at the workload's threshold
    restore()
    kb.block_norms(ctx, cache)
    n_pairs = 4096
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.MASTER_SEED)
    pairs = torch.randint(0, rec.n, (n_pairs, 2), generator=gen, dtype=torch.int32).to(dev)
    cosb = kb.pair_cosines(ctx, cache, pairs)
    torch.cuda.synchronize()
    sev[0].record()
    for _ in range(3):
        kb.pair_cosines(ctx, cache, pairs, out=cosb)
    sev[1].record()
    torch.cuda.synchronize()
    ms_pairs = sev[0].elapsed_time(sev[1]) / 3
    mom = kb.cosine_moments(ctx, cosb).mean(0).cpu()
    mu_s, sigma_s = float(mom[0]), float(mom[1]) ** 0.5
    cross_pairs = (rec.n * rec.n - int((rec.leaf_count.astype("int64") ** 2).sum())) / 2

    # variants of the method, outside the timed steps: the row-order reading of the threshold line, the tree over
    # the requests in ascending length (only where that changes the order), and the "replicate" evaluation mode
    variants = {}
    todo = [("first_row" if rule == kb.RULE_ARGMAX else "argmax", kb.RULE_FIRST_ROW if rule == kb.RULE_ARGMAX else kb.RULE_ARGMAX, plan)]
    sf_spec, sf_order = kb.tree_spec_shortest_first(spec)
    if sf_order.tolist() != sorted(sf_order.tolist()):
        todo.append(("shortest_first", rule, kb.Plan(ctx, cache, sf_spec, args.cand_cap)))
    for name, vrule, vplan in todo:
        restore()
        kb.set_assign_rule(ctx, vplan, vrule)
        vst = kb.fuse_tree(ctx, vplan, rec.thr, want_stats=True, want_timing=True)
        variants[name] = {"fuse_ms": vst.ms_total, "similarity_ms": vst.ms_similarity, "assign_ms": vst.ms_assign,
                          "merge_ms": vst.ms_merge, "compression_ratio": vst.compression_ratio, "fused": vst.fused,
                          "refined_fp64": vst.refined}
        del vplan
    kb.set_assign_rule(ctx, plan, rule)
    restore()
    kb.fuse_tree(ctx, plan, rec.thr, want_stats=True)
    sev[0].record()
    kb.replicate_rescaled(ctx, cache, bt0)
    sev[1].record()
    torch.cuda.synchronize()
    variants["replicate_rescaled"] = {"ms": sev[0].elapsed_time(sev[1]), "blocks_rewritten_at_least": stats.fused,
                                      "includes": "scatter of scale * representative for K and V, table restore, norm pass"}

    # The opt-in prefix screen (an exact shortcut: similarity over the first quarter of every key block + a bound on the
    # tails, every candidate evaluated in full in fp64).  Measured outside the timed steps; the tables must be the same.
    prefix_screen = None
    if not args.screen_prefix and rec.r >= 512:
        restore()
        ref_st = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True)          # the full-length screen on the same input
        bt_ref, k_ref = cache.bt.clone(), cache.K.clone()
        fused_ref = ref_st.fused
        pfx = rec.r // 4
        kb.set_screen_prefix(ctx, plan, pfx)
        best = None
        for _ in range(3):
            restore()
            torch.cuda.synchronize()
            pst = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True, want_timing=True)
            if best is None or pst.ms_total < best.ms_total:
                best = pst
        same = bool(torch.equal(cache.bt, bt_ref)) and bool(torch.equal(cache.K, k_ref)) and best.fused == fused_ref
        del bt_ref, k_ref
        ms_equiv = best.ms_total + stage["decode"] / max(args.steps, 1)
        prefix_screen = {"prefix_elements": pfx, "block_elements": rec.r, "fuse_ms": best.ms_total, "similarity_ms": best.ms_similarity,
                         "assign_ms": best.ms_assign, "merge_ms": best.ms_merge, "norms_ms": best.ms_norms,
                         "refined_fp64": best.refined, "cand_overflow": best.cand_overflow,
                         "tables_and_fused_keys_equal_to_full_screen": same,
                         "executed_similarity_TFLOPs": best.sim_flops * pfx / rec.r / (best.ms_similarity * 1e-3) / 1e12,
                         "step_ms_with_decode": ms_equiv, "blocks_per_s_with_decode": rec.G * rec.n / (ms_equiv * 1e-3),
                         "note": "opt-in (kvfuse_plan_set_screen_prefix); not used in the timed steps, `value` and `roofline`"}
        kb.set_screen_prefix(ctx, plan, 0)

    # The opt-in fp8 screen (the other exact shortcut: similarity over one-byte e4m3 copies of the unit key blocks on the fp8
    # matrix cores + each copy's measured error as a bound; candidates the bound cannot settle are evaluated in fp64).
    # Measured outside the timed steps; the tables must be the same.
    fp8_screen = None
    if not args.screen_fp8 and not args.screen_prefix and rec.r % 64 == 0 and rec.r >= 128:
        restore()
        ref_st = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True)
        bt_ref, k_ref = cache.bt.clone(), cache.K.clone()
        kb.set_screen_fp8(ctx, plan)
        best = None
        for _ in range(3):
            restore()
            torch.cuda.synchronize()
            qst = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True, want_timing=True)
            if best is None or qst.ms_total < best.ms_total:
                best = qst
        same = bool(torch.equal(cache.bt, bt_ref)) and bool(torch.equal(cache.K, k_ref)) and best.fused == ref_st.fused
        err = plan.k8_err[plan.k8_err > 0]
        ms_equiv = best.ms_total + stage["decode"] / max(args.steps, 1)
        eff = best.sim_flops / (best.ms_similarity * 1e-3) / 1e12
        fp8_screen = {"fuse_ms": best.ms_total, "similarity_ms": best.ms_similarity, "assign_ms": best.ms_assign,
                      "merge_ms": best.ms_merge, "norms_ms": best.ms_norms, "refined_fp64": best.refined,
                      "cand_overflow": best.cand_overflow, "tables_and_fused_keys_equal_to_full_screen": same,
                      "similarity_TFLOPs": eff, "frac_of_fp8_peak_5000": eff / 5000.0, "frac_of_bf16_peak_2500": eff / 2500.0,
                      "copy_error_mean": float(err.mean()) if err.numel() else 0.0,
                      "copy_error_max": float(err.max()) if err.numel() else 0.0,
                      "extra_device_bytes": int(plan.k8.numel() + plan.k8_side.numel() * 4),
                      "step_ms_with_decode": ms_equiv, "blocks_per_s_with_decode": rec.G * rec.n / (ms_equiv * 1e-3),
                      "note": "opt-in (kvfuse_plan_set_screen_fp8); not used in the timed steps, `value` and `roofline`"}
        if rec.r // 4 >= 128 and (rec.r // 4) % 64 == 0:
            # both shortcuts together: the product over the first quarter of the copies
            kb.set_screen_prefix(ctx, plan, rec.r // 4)
            best2 = None
            for _ in range(3):
                restore()
                torch.cuda.synchronize()
                bst = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True, want_timing=True)
                if best2 is None or bst.ms_total < best2.ms_total:
                    best2 = bst
            same2 = bool(torch.equal(cache.bt, bt_ref)) and bool(torch.equal(cache.K, k_ref)) and best2.fused == ref_st.fused
            ms2 = best2.ms_total + stage["decode"] / max(args.steps, 1)
            fp8_screen["with_quarter_prefix"] = {
                "fuse_ms": best2.ms_total, "similarity_ms": best2.ms_similarity, "assign_ms": best2.ms_assign,
                "merge_ms": best2.ms_merge, "norms_ms": best2.ms_norms, "refined_fp64": best2.refined,
                "tables_and_fused_keys_equal_to_full_screen": same2,
                "step_ms_with_decode": ms2, "blocks_per_s_with_decode": rec.G * rec.n / (ms2 * 1e-3)}
            kb.set_screen_prefix(ctx, plan, 0)
        # the same with each group's common key direction taken out of the copies first (on this input the keys share
        # none, so this shows what the extra arithmetic costs), ...
        def timed_fuse(k_in=None, runs=3):
            best_t = None
            for _ in range(runs):
                restore()
                if k_in is not None:
                    cache.K.copy_(k_in)
                torch.cuda.synchronize()
                t_st = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True, want_timing=True)
                if best_t is None or t_st.ms_total < best_t.ms_total:
                    best_t = t_st
            return best_t

        def brief(st, **more):
            return dict({"fuse_ms": st.ms_total, "similarity_ms": st.ms_similarity, "assign_ms": st.ms_assign,
                         "merge_ms": st.ms_merge, "norms_ms": st.ms_norms, "fused": st.fused, "refined_fp64": st.refined,
                         "cand_overflow": st.cand_overflow}, **more)

        kb.set_screen_fp8(ctx, plan, centre=True)
        cst = timed_fuse()
        same_c = bool(torch.equal(cache.bt, bt_ref)) and bool(torch.equal(cache.K, k_ref)) and cst.fused == ref_st.fused
        cerr = plan.k8_err[plan.k8_err > 0]
        fp8_screen["centred"] = brief(cst, tables_and_fused_keys_equal_to_full_screen=same_c,
                                      copy_error_mean=float(cerr.mean()) if cerr.numel() else 0.0)
        del k_ref
        if args.common_direction:
            # ... and all three screens on keys that do share one: every key block of a group gets the same random offset of
            # 2.35 times the keys' own spread, which puts unrelated blocks at a cosine of about 0.85: within the plain copies'
            # error bound (0.054 for a pair) of the threshold 0.9, outside that of the centred ones (0.02).  Still closer to
            # the threshold (0.87 and up) the centred copies overflow their lists as well and only the full product is fast.
            gen = torch.Generator(device="cpu")
            gen.manual_seed(2601)
            mu = (2.35 * torch.randn(rec.G, 1, rec.r, generator=gen)).to(dev)
            k_common = torch.empty_like(K0)
            for g0 in range(0, rec.G, 16):
                k_common[g0:g0 + 16] = (K0[g0:g0 + 16].float() + mu[g0:g0 + 16]).to(K0.dtype)
            common = {"recipe": "every key block of group g + 2.35 * N(0, 1)[t * d] drawn once per group"}
            kb.set_screen_fp8(ctx, plan, False)
            fst = timed_fuse(k_common)
            bt_c, k_c = cache.bt.clone(), cache.K.clone()
            common["full_product"] = brief(fst)
            for name, centre in (("fp8_copies", False), ("fp8_copies_centred", True)):
                kb.set_screen_fp8(ctx, plan, centre=centre)
                xst = timed_fuse(k_common, runs=2)
                xerr = plan.k8_err[plan.k8_err > 0]
                common[name] = brief(xst, copy_error_mean=float(xerr.mean()) if xerr.numel() else 0.0,
                                     tables_and_fused_keys_equal_to_full_screen=bool(torch.equal(cache.bt, bt_c)) and
                                     bool(torch.equal(cache.K, k_c)) and xst.fused == fst.fused)
            fp8_screen["keys_with_a_common_direction"] = common
            del bt_c, k_c, k_common, mu
        del bt_ref
        kb.set_screen_fp8(ctx, plan, False)

    # The same step (fusion without the statistics read-back + decode) recorded once in a HIP graph on a stream of
    # its own and replayed: what a serving loop pays per step when the ~45 launches are issued by the graph instead
    # of by the host.  Outside the timed steps; tables must equal those of the eager call.
    graph_replay = None
    if not args.no_graph:
        side = torch.cuda.Stream(dev)
        restore()
        ref_st = kb.fuse_tree(ctx, plan, rec.thr, want_stats=True)
        bt_ref = cache.bt.clone()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            gctx = kb.Context(dev, stream=side)
            gplan = kb.Plan(gctx, cache, spec, args.cand_cap)
            kb.set_assign_rule(gctx, gplan, rule)

            def gstep():
                kb.fuse_tree(gctx, gplan, rec.thr, want_stats=False)
                kb.paged_decode_attn(gctx, cache, rec.kv_heads, q, rs, cl, max_blocks, workspace=ws, out=out)

            restore()
            gstep()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            restore()
            with torch.cuda.graph(graph, stream=side):
                gstep()
            gev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            g_ms = []
            for _ in range(max(args.steps, 1)):
                restore()
                side.synchronize()
                gev[0].record(side)
                graph.replay()
                gev[1].record(side)
                side.synchronize()
                g_ms.append(gev[0].elapsed_time(gev[1]))
            g_same = bool(torch.equal(cache.bt, bt_ref))
            graph_replay = {"ms_per_step": sum(g_ms) / len(g_ms), "replays": len(g_ms),
                            "blocks_per_s": rec.G * rec.n / (sum(g_ms) / len(g_ms) * 1e-3),
                            "tables_equal_to_eager": g_same, "fused_eager": ref_st.fused,
                            "note": "fusion (no statistics read-back) + decode as one HIP graph; not used in `value`"}
            del graph, gplan, gctx
        del bt_ref
        torch.cuda.synchronize()

    # decode attention over the un-fused cache (logical = physical bytes): the clean HBM figure of the decode kernel
    restore()
    cache.identity_scales()
    kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, max_blocks, workspace=ws, out=out)
    torch.cuda.synchronize()
    sev[0].record()
    for _ in range(3):
        kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, max_blocks, workspace=ws, out=out)
    sev[1].record()
    torch.cuda.synchronize()
    ms_dec_unfused = sev[0].elapsed_time(sev[1]) / 3

    # what the machine sustains, measured with the library's own probes after the timed steps (they load the chip
    # heavily and would otherwise warm it up for the steps): the MFMA instruction of the similarity kernel on
    # random and on constant operands, and a plain device copy
    blk_bytes_probe = rec.r * (2 if rec.dtype == torch.bfloat16 else 4)
    probes = {"mfma_bf16_random_operands_TFLOPs": kp.mfma_bf16(True, dev),
              "mfma_bf16_constant_operands_TFLOPs": kp.mfma_bf16(False, dev),
              "mfma_fp8_random_operands_TFLOPs": kp.mfma_fp8(True, dev),
              "mfma_fp8_constant_operands_TFLOPs": kp.mfma_fp8(False, dev),
              "tile_loop_bf16_TFLOPs": kp.tile_loop_bf16(K0, True) if rec.dtype == torch.bfloat16 else None,
              "tile_loop_bf16_no_loads_TFLOPs": kp.tile_loop_bf16(K0, False) if rec.dtype == torch.bfloat16 else None,
              "copy_kernel_GBps": kp.copy(K0, cache.K, repeats=3),
              "read2_write1_GBps": kp.read2_write1(cache.K, blk_bytes_probe, repeats=3)}
    k = max(args.steps, 1)
    stage = {a: b / k for a, b in stage.items()}
    ms_step = sum(walls) / k
    ms_median = sorted(walls)[len(walls) // 2] if walls else 0.0
    blocks = rec.G * rec.n
    elem = 2 if rec.dtype == torch.bfloat16 else 4
    blk_bytes = rec.r * elem
    sim_tflops = stats.sim_flops / (stage["similarity"] * 1e-3) / 1e12 if stage["similarity"] > 0 else 0.0
    peak = 2500.0 if rec.dtype == torch.bfloat16 else 157.3
    phys_bytes = stats.physical_blocks * blk_bytes * 2
    logi_bytes = stats.logical_blocks * blk_bytes * 2
    traffic = None      # HBM bytes per similarity launch, from the committed rocprofv3 counter summary of this workload
    prof = os.path.join(ROOT, "profiles", f"{rec.name}_kernels.md")
    if args.workload == rec.name and os.path.exists(prof):
        for ln in open(prof):
            if ln.startswith("traffic_bytes_per_similarity_launch"):
                traffic = float(ln.split("=")[1].split()[0])
    line = {
        "metric": "KV blocks fused/sec (+ % MFMA peak); fused-table decode attn HBM GB/s",
        "value": blocks / (ms_step * 1e-3),
        "unit": "blocks/s",
        "value_is": "logical KV blocks (one per layer, KV head and block position) through norms, the whole fusion tree and "
                    "one decode-attention step, per second; blocks that fusion evicted per second are in blocks_fused_per_s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "ms_per_step_median": ms_median,
        "request_level_blocks_per_s": blocks / (rec.layers * rec.kv_heads) / (ms_step * 1e-3),
        "blocks_fused_per_s": stats.fused / (ms_step * 1e-3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if rec.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": f"{rec.name}: {rec.layers} layers x {rec.kv_heads} KV heads, d {rec.d}, block {rec.t}, "
                               f"{rec.B} requests, {rec.n} logical blocks per group, thr {rec.thr}",
                   "groups": rec.G, "logical_blocks": blocks, "physical_blocks_after": stats.physical_blocks,
                   "compression_ratio": stats.compression_ratio, "fused": stats.fused,
                   "near_threshold": stats.near_threshold, "refined_fp64": stats.refined,
                   "cand_overflow": stats.cand_overflow, "tree_heights": stats.n_heights,
                   "assign_rule": args.assign_rule, "shortest_first": bool(args.shortest_first)},
        "stages_ms": stage,
        "decode": {"ms": stage["decode"], "physical_GBps": phys_bytes / (stage["decode"] * 1e-3) / 1e9,
                   "logical_GBps": logi_bytes / (stage["decode"] * 1e-3) / 1e9, "hbm_peak_GBps": 8000.0,
                   "frac_of_hbm_peak_physical": phys_bytes / (stage["decode"] * 1e-3) / 1e9 / 8000.0},
        "decode_unfused": {"ms": ms_dec_unfused, "GBps": logi_bytes / (ms_dec_unfused * 1e-3) / 1e9,
                           "frac_of_hbm_peak": logi_bytes / (ms_dec_unfused * 1e-3) / 1e9 / 8000.0,
                           "note": "same kernel and queries on the cache before fusion: logical = physical bytes"},
        "decode_shared_blocks": {"ms": ms_shared, "physical_GBps": phys_bytes / (ms_shared * 1e-3) / 1e9,
                                 "max_abs_diff_vs_decode": shared_diff, "plan_build_s": t_plan, "clusters": si.clusters,
                                 "logical_blocks": si.logical_blocks, "served_through_clusters": si.shared_instances,
                                 "block_reads": si.cluster_block_reads + si.residual_block_reads,
                                 "plan_device_MB": si.device_bytes / 1e6},
        "prefill_with_reuse": prefill,
        "threshold_stats": {"pairs_per_group": n_pairs, "pair_cosines_ms": ms_pairs,
                            "pair_cosines_GBps": rec.G * n_pairs * 2 * blk_bytes / (ms_pairs * 1e-3) / 1e9,
                            "mean_cosine": mu_s, "sigma_cosine": sigma_s,
                            "gaussian_exceedance_rate_per_group_at_thr": kb.exceedance_rate(cross_pairs, mu_s, sigma_s, rec.thr),
                            "note": "the synthetic cache plants exact and near duplicates, which a Gaussian fit of the "
                                    "bulk does not see; the rate is shown for the mechanism, not as a forecast"},
        "merge": {"ms": stage["merge"], "targets": stats.merge_targets, "members": stats.fused,
                  "algorithmic_bytes": (2 * stats.merge_targets + stats.fused) * blk_bytes * 2,
                  "GBps": (2 * stats.merge_targets + stats.fused) * blk_bytes * 2 / (stage["merge"] * 1e-3) / 1e9,
                  "frac_of_hbm_peak": (2 * stats.merge_targets + stats.fused) * blk_bytes * 2 / (stage["merge"] * 1e-3) / 1e9 / 8000.0,
                  "frac_of_read2_write1_probe": (2 * stats.merge_targets + stats.fused) * blk_bytes * 2 / (stage["merge"] * 1e-3) / 1e9
                                                / probes["read2_write1_GBps"]},
        "variants": variants,
        "prefix_screen": prefix_screen,
        "fp8_screen": fp8_screen,
        "graph_replay": graph_replay,
        "norms": {"ms": stage["norms"], "GBps": logi_bytes / (stage["norms"] * 1e-3) / 1e9},
        "roofline": {"kernel": "similarity_ring_kernel (256 x 256 tile instance on the upper heights, 128 x 128 on the lowest)",
                     "bound": "mfma", "achieved": sim_tflops, "peak": peak,
                     "unit": "TFLOP/s", "frac": sim_tflops / peak, "traffic": traffic,
                     "frac_of_measured_mfma_rate": (sim_tflops / probes["mfma_bf16_random_operands_TFLOPs"]
                                                    if rec.dtype == torch.bfloat16 else None),
                     "frac_of_stripped_tile_loop": (sim_tflops / probes["tile_loop_bf16_TFLOPs"]
                                                    if rec.dtype == torch.bfloat16 else None),
                     "launches_per_step": stats.n_heights,
                     "flops_per_step": stats.sim_flops, "ms_per_step": stage["similarity"]},
        "machine_probes": probes,
        "generation_s": t_gen,
    }
    if args.per_height:
        line["per_height"] = per_height_table(kb, ctx, cache, plan, rec, restore, rec.thr)
    if args.power:
        line["power"] = power_report(kb, kp, ctx, cache, plan, rec, restore, torch,
                                     decode_step=lambda: kb.paged_decode_attn(ctx, cache, rec.kv_heads, q, rs, cl, max_blocks,
                                                                              workspace=ws, out=out))
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, reduced=args.cpu_baseline_reduced)
    print(json.dumps(line))
    sys.stdout.flush()
    # nothing of this run may outlive it: no worker process is started on purpose, and none is left behind
    try:
        import psutil
        for child in psutil.Process().children(recursive=True):
            print(f"bench.py: ending left-over child process {child.pid} ({child.name()})", file=sys.stderr)
            child.terminate()
    except Exception:
        pass


if __name__ == "__main__":
    main()
