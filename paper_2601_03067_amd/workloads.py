"""Seeded synthetic inputs for the Fast Fusion hot path.

This module only draws random numbers and lays out tables; it holds none of the
method's arithmetic (no norms, similarities, fusion or attention) and is the one
piece that the tests hand to both the HIP library and the CPU oracle.

The paper evaluates on vLLM's random-data benchmark and on Llama / Qwen KV caches of real
datasets (results section); neither weights nor datasets are available, so these
generators stand in for them: same tensor shapes (layers x KV heads groups, tokens per
block, head size), same structure (shared prefixes, near-duplicate blocks across requests
or chunks, ragged lengths), values i.i.d. normal.

A workload is described by a *recipe* shared by all groups -- for every logical block either
"fresh random" or "base block ``src`` plus N(0, sigma) noise" (sigma 0 = exact copy) -- and is
materialised group by group from per-group seeds, so any subset of groups can be regenerated
bit-identically on any device of the same kind.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

MASTER_SEED = 20260103


def _subseed(*parts: int) -> int:
    """Deterministic 63-bit mix of small integers (splitmix-style), independent of PYTHONHASHSEED."""
    x = 0x9E3779B97F4A7C15
    for p in parts:
        x = (x ^ (int(p) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2))) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


@dataclass
class Recipe:
    """Structure of one workload; identical for every (layer, KV head) group."""

    name: str
    config_id: int
    layers: int
    kv_heads: int
    q_heads: int
    t: int                      # tokens per block
    d: int                      # head size
    dtype: torch.dtype
    thr: float
    # per logical block (length n)
    src: np.ndarray             # int64: base index, or -1 for a fresh random block
    sigma: np.ndarray           # float32: noise std added to the base (0 = exact copy)
    n_base: int
    # requests: logical range [req_start[b], req_start[b] + req_blocks[b]); last block may be partial
    req_start: np.ndarray       # int32 [B]
    req_blocks: np.ndarray      # int32 [B]
    ctx_len: np.ndarray         # int32 [B] tokens
    # fusion leaves (full blocks only) and units (requests) over leaves
    leaf_start: np.ndarray      # int32 [n_leaves]
    leaf_count: np.ndarray      # int32 [n_leaves]
    unit_leaf_ptr: np.ndarray   # int32 [n_units + 1]
    group_size: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.layers * self.kv_heads

    @property
    def r(self) -> int:
        return self.t * self.d

    @property
    def n(self) -> int:
        return int(len(self.src))

    @property
    def B(self) -> int:
        return int(len(self.req_start))


def _bff_leaves(req_start, req_full):
    """One leaf per request holding its full blocks; one unit per request."""
    leaf_start = np.asarray(req_start, np.int32)
    leaf_count = np.asarray(req_full, np.int32)
    unit_leaf_ptr = np.arange(len(req_start) + 1, dtype=np.int32)
    return leaf_start, leaf_count, unit_leaf_ptr


def _chunk_leaves(req_start, req_full, chunk_blocks):
    """Each request is a unit; its leaves are runs of ``chunk_blocks`` full blocks (last may be short)."""
    ls, lc, up = [], [], [0]
    for s, f in zip(req_start, req_full):
        off = 0
        while off < f:
            c = min(chunk_blocks, f - off)
            ls.append(s + off)
            lc.append(c)
            off += c
        up.append(len(ls))
    return np.asarray(ls, np.int32), np.asarray(lc, np.int32), np.asarray(up, np.int32)


# ----------------------------------------------------------------------
# the five configurations (sizes are parameters so that tests can shrink them)
# ----------------------------------------------------------------------

def tiny_bff(seed: int = MASTER_SEED) -> Recipe:
    """Config 1: 1 layer, 2 KV heads, d 64, t 16, 4 requests x 8 blocks, fp32, thr 0.95.

    Ten disjoint source->copy pairs across different requests: 8 noisy (sigma 0.01), 2 exact.
    Every request decodes one query over its 128 tokens."""
    rng = np.random.default_rng(_subseed(seed, 1, 0))
    n_req, p = 4, 8
    n = n_req * p
    perm = rng.permutation(n)
    src = np.full(n, -1, np.int64)
    sigma = np.zeros(n, np.float32)
    used = np.zeros(n, bool)
    pairs = []
    for x in perm:
        if len(pairs) == 10:
            break
        if used[x]:
            continue
        cands = [y for y in perm if not used[y] and y // p != x // p and y != x]
        if not cands:
            continue
        y = cands[0]
        used[x] = used[y] = True
        pairs.append((int(x), int(y)))
    for k, (a, b) in enumerate(pairs):
        src[a] = k
        src[b] = k
        sigma[b] = 0.01 if k < 8 else 0.0
    req_start = np.arange(n_req, dtype=np.int32) * p
    req_blocks = np.full(n_req, p, np.int32)
    ls, lc, up = _bff_leaves(req_start, req_blocks)
    return Recipe("tiny_bff", 1, 1, 2, 4, 16, 64, torch.float32, 0.95, src, sigma, len(pairs), req_start,
                  req_blocks, req_blocks * 16, ls, lc, up, notes={"pairs": pairs, "expected_physical": n - len(pairs)})


def llama8b_bff(n_req: int = 64, tokens: int = 2048, layers: int = 32, kv_heads: int = 8, prefix_tokens: int = 512,
                near_frac: float = 0.25, near_pool: int = 512, sigma: float = 0.05, t: int = 16, d: int = 128,
                dtype=torch.bfloat16, seed: int = MASTER_SEED) -> Recipe:
    """Config 2: Llama-3-8B-shaped BFF.  Every request = the same prefix blocks (exact) + random blocks, of which
    ``near_frac`` are ``base[u] + N(0, sigma)`` with u uniform over a pool of ``near_pool`` bases.  thr 0.9."""
    rng = np.random.default_rng(_subseed(seed, 2, 0))
    p = tokens // t
    pre = prefix_tokens // t
    n = n_req * p
    src = np.full(n, -1, np.int64)
    sg = np.zeros(n, np.float32)
    n_near = int(round((p - pre) * near_frac))
    for b in range(n_req):
        base = b * p
        src[base: base + pre] = np.arange(pre)
        pos = rng.choice(p - pre, size=n_near, replace=False) + pre
        src[base + pos] = pre + rng.integers(0, near_pool, size=n_near)
        sg[base + pos] = sigma
    req_start = np.arange(n_req, dtype=np.int32) * p
    req_blocks = np.full(n_req, p, np.int32)
    ls, lc, up = _bff_leaves(req_start, req_blocks)
    return Recipe("llama8b_bff", 2, layers, kv_heads, 4 * kv_heads, t, d, dtype, 0.9, src, sg, pre + near_pool,
                  req_start, req_blocks, np.full(n_req, tokens, np.int32), ls, lc, up)


def cff_long(tokens: int = 32768, chunk_tokens: int = 2048, layers: int = 32, kv_heads: int = 8, reuse: float = 0.4,
             sigma: float = 0.05, t: int = 16, d: int = 128, dtype=torch.bfloat16, seed: int = MASTER_SEED) -> Recipe:
    """Config 3: one long request split into chunks; each chunk after the first takes ``reuse`` of its blocks
    from uniformly drawn earlier blocks (their origin + N(0, sigma)).  CFF across chunks, thr 0.9."""
    rng = np.random.default_rng(_subseed(seed, 3, 0))
    p = tokens // t
    cb = chunk_tokens // t
    src = np.full(p, -1, np.int64)
    sg = np.zeros(p, np.float32)
    n_base = 0
    for c in range(1, (p + cb - 1) // cb):
        lo, hi = c * cb, min((c + 1) * cb, p)
        k = int(round((hi - lo) * reuse))
        pos = rng.choice(hi - lo, size=k, replace=False) + lo
        for x in pos:
            y = int(rng.integers(0, lo))
            if src[y] < 0:          # promote the origin to a base block (value = the base, exactly)
                src[y] = n_base
                n_base += 1
            src[x] = src[y]
            sg[x] = sigma
    req_start = np.zeros(1, np.int32)
    req_blocks = np.array([p], np.int32)
    ls, lc, up = _chunk_leaves(req_start, req_blocks, cb)
    return Recipe("cff_long", 3, layers, kv_heads, 4 * kv_heads, t, d, dtype, 0.9, src, sg, max(n_base, 1), req_start,
                  req_blocks, np.array([tokens], np.int32), ls, lc, up)


def zipf_bff(n_req: int = 256, tokens: int = 4096, layers: int = 80, kv_heads: int = 8, pool: int = 20000,
             a: float = 1.1, sigma: float = 0.03, t: int = 32, d: int = 128, thr: float = 0.9,
             dtype=torch.bfloat16, seed: int = MASTER_SEED) -> Recipe:
    """Config 4: every block = base[z] + N(0, sigma), z ~ Zipf(a) truncated to ``pool`` ranks."""
    rng = np.random.default_rng(_subseed(seed, 4, 0))
    p = tokens // t
    n = n_req * p
    w = 1.0 / np.arange(1, pool + 1, dtype=np.float64) ** a
    w /= w.sum()
    src = rng.choice(pool, size=n, p=w).astype(np.int64)
    sg = np.full(n, sigma, np.float32)
    req_start = np.arange(n_req, dtype=np.int32) * p
    req_blocks = np.full(n_req, p, np.int32)
    ls, lc, up = _bff_leaves(req_start, req_blocks)
    return Recipe("zipf_bff", 4, layers, kv_heads, 8 * kv_heads, t, d, dtype, thr, src, sg, pool, req_start,
                  req_blocks, np.full(n_req, tokens, np.int32), ls, lc, up)


def mixed(n_req: int = 512, min_tokens: int = 512, max_tokens: int = 8192, chunk_tokens: int = 2048, layers: int = 32,
          kv_heads: int = 8, exact_frac: float = 0.10, near_frac: float = 0.30, pool: int = 4096, sigma: float = 0.05,
          t: int = 16, d: int = 128, dtype=torch.bfloat16, seed: int = MASTER_SEED) -> Recipe:
    """Config 5: ragged requests (uniform lengths, partial tail blocks), chunked; per full block 10 % exact copies
    of a pool block, 30 % noisy copies, rest random.  Chunks of a request fuse first, then requests (thr 0.9)."""
    rng = np.random.default_rng(_subseed(seed, 5, 0))
    lens = rng.integers(min_tokens, max_tokens + 1, size=n_req)
    full = lens // t
    blocks = (lens + t - 1) // t
    req_start = np.concatenate([[0], np.cumsum(blocks)[:-1]]).astype(np.int32)
    n = int(blocks.sum())
    src = np.full(n, -1, np.int64)
    sg = np.zeros(n, np.float32)
    for b in range(n_req):
        u = rng.random(full[b])
        z = rng.integers(0, pool, size=full[b])
        xs = req_start[b] + np.arange(full[b])
        ex = u < exact_frac
        nr = (u >= exact_frac) & (u < exact_frac + near_frac)
        src[xs[ex]] = z[ex]
        src[xs[nr]] = z[nr]
        sg[xs[nr]] = sigma
    ls, lc, up = _chunk_leaves(req_start, full.astype(np.int32), chunk_tokens // t)
    return Recipe("mixed", 5, layers, kv_heads, 4 * kv_heads, t, d, dtype, 0.9, src, sg, pool, req_start,
                  blocks.astype(np.int32), lens.astype(np.int32), ls, lc, up)


# ----------------------------------------------------------------------
# materialisation
# ----------------------------------------------------------------------

def group_values(rec: Recipe, g: int, kind: int, device, seed: int = MASTER_SEED, rows_per_pass: int = 16384) -> torch.Tensor:
    """Values [n][r] of group ``g`` (kind 0 = K, 1 = V) in the recipe's dtype, on ``device``."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(_subseed(seed, rec.config_id, g, kind))
    r, n = rec.r, rec.n
    base = torch.randn(rec.n_base, r, generator=gen, device=dev, dtype=torch.float32)
    out = torch.empty(n, r, device=dev, dtype=rec.dtype)
    src = torch.from_numpy(rec.src).to(dev)
    sg = torch.from_numpy(rec.sigma).to(dev)
    for lo in range(0, n, rows_per_pass):
        hi = min(n, lo + rows_per_pass)
        x = torch.randn(hi - lo, r, generator=gen, device=dev, dtype=torch.float32)
        s = src[lo:hi]
        planted = s >= 0
        if bool(planted.any()):
            b = base[s.clamp(min=0)]
            x = torch.where(planted[:, None], b + sg[lo:hi, None] * x, x)
        out[lo:hi] = x.to(rec.dtype)
    return out


def materialise(rec: Recipe, device, groups=None, seed: int = MASTER_SEED, phys_perm: bool = False):
    """Build pools and tables for ``groups`` (default: all) -> dict of tensors.

    K, V   [Gsel][P][r] in rec.dtype, P = n (one physical block per logical block before fusion)
    bt     [Gsel][n] int32: identity, or a seeded permutation per group when ``phys_perm`` (paged layout)
    q      [layers_sel... ] not built here; see ``queries``.
    """
    groups = list(range(rec.G)) if groups is None else list(groups)
    dev = torch.device(device)
    n, r = rec.n, rec.r
    K = torch.empty(len(groups), n, r, device=dev, dtype=rec.dtype)
    V = torch.empty(len(groups), n, r, device=dev, dtype=rec.dtype)
    bt = torch.empty(len(groups), n, device=dev, dtype=torch.int32)
    for i, g in enumerate(groups):
        k = group_values(rec, g, 0, dev, seed)
        v = group_values(rec, g, 1, dev, seed)
        if phys_perm:
            perm = torch.from_numpy(np.random.default_rng(_subseed(seed, rec.config_id, g, 7)).permutation(n)).to(dev)
            K[i][perm] = k
            V[i][perm] = v
            bt[i] = perm.to(torch.int32)
        else:
            K[i] = k
            V[i] = v
            bt[i] = torch.arange(n, device=dev, dtype=torch.int32)
    return {"K": K, "V": V, "bt": bt, "groups": groups}


def queries(rec: Recipe, device, layers=None, seed: int = MASTER_SEED) -> torch.Tensor:
    """Decode queries [len(layers)][B][Hq][d] ~ N(0,1) in the recipe's dtype."""
    layers = list(range(rec.layers)) if layers is None else list(layers)
    dev = torch.device(device)
    out = torch.empty(len(layers), rec.B, rec.q_heads, rec.d, device=dev, dtype=rec.dtype)
    for i, l in enumerate(layers):
        gen = torch.Generator(device=dev)
        gen.manual_seed(_subseed(seed, rec.config_id, l, 2))
        out[i] = torch.randn(rec.B, rec.q_heads, rec.d, generator=gen, device=dev, dtype=torch.float32).to(rec.dtype)
    return out


def to_numpy_pool(x: torch.Tensor) -> np.ndarray:
    """Device tensor -> host numpy; bfloat16 becomes its uint16 bit pattern (numpy has no bfloat16)."""
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()
