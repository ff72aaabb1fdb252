"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

The paper prints no numeric walk-through of Algorithm 1, so the pins are closed forms, invariants,
special cases that reduce to textbook routines, planted structure with a known answer, and an
independently written dense brute force on tiny inputs.
"""
import math

import numpy as np
import pytest
import torch

from paper_2601_03067_amd import workloads as wl


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.asarray(x32, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _identity_setup(K, V, leaves):
    """Leaves = list of block counts; identity table."""
    n = K.shape[0]
    bt = np.arange(n, dtype=np.int32)
    lc = np.asarray(leaves, np.int32)
    ls = np.concatenate([[0], np.cumsum(lc)[:-1]]).astype(np.int32)
    up = np.arange(len(leaves) + 1, dtype=np.int32)
    return bt, ls, lc, up


# ---------------------------------------------------------------- rounding rule

def test_bf16_rounding_matches_library_conversion_and_has_no_double_rounding(oracle):
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.standard_normal(2000), rng.standard_normal(200) * 1e-3, rng.standard_normal(200) * 1e4,
                         [0.0, 1.0, -1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 2.0 ** -130, 3.0e38]])
    xs32 = xs.astype(np.float32)          # exactly representable in binary32: torch's RNE conversion is the reference
    want = torch.from_numpy(xs32).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_bf16(float(x)) for x in xs32])
    assert np.array_equal(got, want)
    # ties go to even
    assert oracle.round_bf16(1 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6
    # a double that binary32 would first round onto a tie must still round by its true value
    assert oracle.round_bf16(1 + 2.0 ** -8 + 2.0 ** -40) == 1 + 2.0 ** -7
    assert oracle.round_bf16(1 + 2.0 ** -8 - 2.0 ** -40) == 1.0


# ---------------------------------------------------------------- norms and similarity

def test_norms_and_cosine_closed_forms(oracle):
    # 3-4-5 triangles: norms and cosines known exactly
    K = np.array([[3, 4, 0, 0], [0, 0, 5, 12], [6, 8, 0, 0], [4, 3, 0, 0], [0, 0, 0, 0]], np.float32)
    nrm = oracle.block_norms(K)
    assert np.array_equal(nrm, [5, 13, 10, 5, 0])
    S = oracle.similarity(K, nrm, np.array([0, 1, 4]), np.array([2, 3, 1]))
    want = np.array([[1.0, 24 / 25, 0.0], [0.0, 0.0, 1.0], [0.0, 0.0, 0.0]])
    assert np.allclose(S, want, atol=1e-15)
    # not symmetric in its arguments' roles: row = left, column = right
    S2 = oracle.similarity(K, nrm, np.array([2, 3, 1]), np.array([0, 1, 4]))
    assert np.allclose(S2, want.T, atol=1e-15)


def test_similarity_equals_library_matmul_on_unit_vectors(oracle):
    rng = np.random.default_rng(1)
    K = rng.standard_normal((40, 96)).astype(np.float32)
    nrm = oracle.block_norms(K)
    L, R = np.arange(0, 17), np.arange(17, 40)
    S = oracle.similarity(K, nrm, L, R)
    U = K.astype(np.float64) / np.linalg.norm(K.astype(np.float64), axis=1, keepdims=True)
    assert np.allclose(S, U[L] @ U[R].T, atol=1e-13)
    assert np.allclose(nrm, np.linalg.norm(K.astype(np.float64), axis=1), rtol=1e-14)


def test_bf16_pool_is_read_exactly(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 32)).astype(np.float32)
    bits = _bf16_bits(x)
    exact = wl_to_f64(bits)
    nrm = oracle.block_norms(bits)
    assert np.allclose(nrm, np.sqrt((exact ** 2).sum(1)), rtol=1e-15)


def wl_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_gaussian_exceedance_count_matches_analysis_section(oracle):
    """Analysis section: with similarities ~ N(mu, sigma^2) the number above u is about n(1 - Phi((u-mu)/sigma)).
    For i.i.d. normal blocks the cosine is ~ N(0, 1/r), so the count above u over m1*m2 pairs is Poisson-like
    with rate n(1 - Phi(u sqrt(r)))."""
    rng = np.random.default_rng(3)
    r, m = 64, 160
    K = rng.standard_normal((2 * m, r)).astype(np.float32)
    nrm = oracle.block_norms(K)
    S = oracle.similarity(K, nrm, np.arange(m), np.arange(m, 2 * m))
    u = 0.25
    lam = m * m * 0.5 * math.erfc(u * math.sqrt(r) / math.sqrt(2))
    cnt = int((S > u).sum())
    assert abs(cnt - lam) <= 4 * math.sqrt(lam) + 0.12 * lam   # 12 % slack: the cosine of finite-r normals is only ~ normal
    a, best, second = oracle.assign(S, u)
    assert (a >= 0).sum() == int((S.max(0) > u).sum())


# ---------------------------------------------------------------- threshold / arg-max step

def test_assign_strict_threshold_lowest_index_ties(oracle):
    S = np.array([[0.5, 0.9, 0.2, 0.7],
                  [0.9, 0.9, 0.1, 0.7],
                  [0.1, 0.3, 0.2, 0.6999]])
    a, best, second = oracle.assign(S, 0.7)
    assert a.tolist() == [1, 0, -1, -1]          # column 1: tie -> lowest row; column 3: 0.7 > 0.7 is false
    assert best.tolist() == [0.9, 0.9, 0.2, 0.7]
    assert second.tolist() == [0.5, 0.9, 0.2, 0.7]
    a2, _, _ = oracle.assign(S, 1.5)
    assert a2.tolist() == [-1, -1, -1, -1]


# ---------------------------------------------------------------- fusion step: closed forms

def test_two_block_fusion_is_the_bisector(oracle):
    """Two unit directions at cosine s fuse into their bisector: cos(member, rep) = sqrt((1+s)/2)."""
    K = np.array([[1.0, 0.0], [1.5, 2.0]], np.float32)       # b = 2.5 * (0.6, 0.8), cos = 0.6
    V = np.array([[0.0, 3.0], [4.0, 0.0]], np.float32)       # orthogonal values: rep_v = (1,1)/sqrt2
    bt, ls, lc, up = _identity_setup(K, V, [1, 1])
    res = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.5)
    assert res.bt.tolist() == [0, 0]
    rep = res.kpool[0].astype(np.float64)
    assert np.allclose(rep, [2 / math.sqrt(5), 1 / math.sqrt(5)], atol=1e-7)     # (0.894427, 0.447214)
    assert np.allclose(res.vpool[0], [1 / math.sqrt(2), 1 / math.sqrt(2)], atol=1e-7)
    assert np.allclose(res.scale_k, [1.0, 2.5], rtol=1e-6)                      # ||a|| = 1, ||b|| = 2.5, ||rep|| = 1
    assert np.allclose(res.scale_v, [3.0, 4.0], rtol=1e-6)
    assert math.isclose(float(rep @ np.array([0.6, 0.8])), math.sqrt((1 + 0.6) / 2), rel_tol=1e-6)
    assert res.refcount.tolist() == [2, 0] and res.free_list.tolist() == [1]
    assert res.compression_ratio == 2.0
    # below-threshold pair is left alone, byte for byte
    res2 = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.6)                     # cos == thr is not above it
    assert res2.bt.tolist() == [0, 1] and np.array_equal(res2.kpool, K) and np.array_equal(res2.vpool, V)
    assert res2.scale_k.tolist() == [1.0, 1.0]


def test_decisions_near_the_threshold_are_counted_by_their_distance_to_it(oracle):
    """The "reported separately" counter: a decision is near the threshold when its best cosine lies within `band` of
    thr, whichever side it is on.  One left block e1 against right blocks at known angles: cosines thr + 4e-4 and
    thr - 4e-4 (near; the first fuses, the second does not), thr + 3e-3 and thr - 3e-3 (not near), and one exactly
    orthogonal.  The counters and the smallest margin follow by hand."""
    thr, band = 0.9, 1e-3
    cosines = [thr + 4e-4, thr - 4e-4, thr + 3e-3, thr - 3e-3, 0.0]
    K = np.array([[1.0, 0.0]] + [[c, math.sqrt(1.0 - c * c)] for c in cosines], np.float32)
    V = K.copy()
    bt, ls, lc, up = _identity_setup(K, V, [1, len(cosines)])
    res = oracle.fuse_group(K, V, bt, ls, lc, up, thr=thr, band=band)
    decisions, fused, near, ties, min_margin = (res.stats[i] for i in range(5))
    assert (decisions, fused, near, ties) == (5, 2, 2, 0)
    assert res.bt.tolist() == [0, 0, 2, 0, 4, 5]
    assert abs(min_margin - 4e-4) < 1e-6                      # binary32 storage moves a cosine by ~1e-7 at most
    # a wider band takes the +-3e-3 decisions in as well; a narrower one leaves none
    assert oracle.fuse_group(K, V, bt, ls, lc, up, thr=thr, band=5e-3).stats[2] == 4
    assert oracle.fuse_group(K, V, bt, ls, lc, up, thr=thr, band=1e-4).stats[2] == 0


def test_sum_is_over_current_unit_representatives_not_member_mean(oracle):
    """Three leaves a | b | c with a,b fusing first (left subtree = [a], right = [b, c] split as b | c).
    With leaves [a],[b],[c] the tree is FF([a]) vs FF([b],[c]): b and c fuse first, then their unit rep meets a.
    The final direction is normalize(a_hat + normalize(b_hat + c_hat)), not normalize(a_hat + b_hat + c_hat)."""
    ang = np.deg2rad([0.0, 20.0, 40.0])
    K = np.stack([np.cos(ang), np.sin(ang)], 1).astype(np.float32) * np.array([[1.0], [2.0], [3.0]], np.float32)
    V = K.copy()
    bt, ls, lc, up = _identity_setup(K, V, [1, 1, 1])
    res = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.8)
    assert res.bt.tolist() == [0, 0, 0]
    u = lambda t: np.array([math.cos(t), math.sin(t)])
    bc = u(ang[1]) + u(ang[2]); bc /= np.linalg.norm(bc)
    want = u(ang[0]) + bc; want /= np.linalg.norm(want)
    mean3 = u(ang[0]) + u(ang[1]) + u(ang[2]); mean3 /= np.linalg.norm(mean3)
    assert np.allclose(res.kpool[0], want, atol=2e-7)
    assert not np.allclose(res.kpool[0], mean3, atol=1e-3)
    assert np.allclose(res.scale_k, [1.0, 2.0, 3.0], rtol=1e-6)
    assert res.refcount.tolist() == [3, 0, 0]
    assert sorted(res.free_list.tolist()) == [1, 2]


def test_identical_blocks_in_different_leaves_collapse(oracle):
    """Fusion subsumes exact prefix sharing: m identical blocks in m leaves -> one physical block, same direction."""
    rng = np.random.default_rng(5)
    r, m = 48, 6
    base = rng.standard_normal(r).astype(np.float32)
    other = rng.standard_normal((m, r)).astype(np.float32)
    K = np.empty((2 * m, r), np.float32)
    K[0::2] = base
    K[1::2] = other
    V = K[:, ::-1].copy()
    bt, ls, lc, up = _identity_setup(K, V, [2] * m)
    res = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.95)
    assert (res.bt[0::2] == 0).all() and res.refcount[0] == m
    assert res.bt[1::2].tolist() == list(range(1, 2 * m, 2))
    d = res.kpool[0].astype(np.float64)
    assert np.allclose(d, base / np.linalg.norm(base.astype(np.float64)), atol=2e-7)
    assert np.allclose(res.scale_k[0::2], np.linalg.norm(base.astype(np.float64)), rtol=1e-6)
    assert res.n_physical == m + 1 and math.isclose(res.compression_ratio, 2 * m / (m + 1))
    # duplicates inside one leaf are never compared with each other
    bt1, ls1, lc1, up1 = _identity_setup(K, V, [2 * m])
    res1 = oracle.fuse_group(K, V, bt1, ls1, lc1, up1, thr=0.95)
    assert res1.bt.tolist() == list(range(2 * m)) and res1.compression_ratio == 1.0


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_rescaling_blocks_by_powers_of_two_changes_only_the_scales(oracle, kind):
    """Method section: a block is a unit direction plus a norm.  Multiplying every block by its own power of two is
    exact in binary floating point and leaves every direction, hence every cosine, decision and fused representative,
    bit for bit as it was; only the norms, and with them the scales of the logical blocks, pick up the factor."""
    rec = wl.llama8b_bff(n_req=4, tokens=8 * 40, layers=1, kv_heads=1, prefix_tokens=32, near_pool=8, t=8, d=16,
                         dtype=torch.float32 if kind == "f32" else torch.bfloat16)
    m = wl.materialise(rec, "cpu", phys_perm=True)
    K, V, bt = m["K"][0], m["V"][0], m["bt"][0].numpy()
    rng = np.random.default_rng(99)
    fk = torch.from_numpy(2.0 ** rng.integers(-6, 7, size=rec.n)).to(K.dtype)[:, None]
    fv = torch.from_numpy(2.0 ** rng.integers(-6, 7, size=rec.n)).to(K.dtype)[:, None]
    K2, V2 = K * fk, V * fv
    assert torch.equal(K2 / fk, K) and torch.equal(V2 / fv, V)            # the scaling is exact
    a = oracle.fuse_group(wl.to_numpy_pool(K), wl.to_numpy_pool(V), bt, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr)
    b = oracle.fuse_group(wl.to_numpy_pool(K2), wl.to_numpy_pool(V2), bt, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr)
    assert int(a.stats[1]) > 20 and np.array_equal(a.bt, b.bt) and np.array_equal(a.refcount, b.refcount)
    assert np.array_equal(a.stats[:4], b.stats[:4])
    fused = a.refcount > 1                                                # representatives: unit vectors, identical
    assert fused.any() and np.array_equal(a.kpool[fused], b.kpool[fused]) and np.array_equal(a.vpool[fused], b.vpool[fused])
    # logical entry x had its original block at bt[x]: its scale carries that block's factor wherever it points now
    fkx, fvx = fk.double().numpy()[bt, 0], fv.double().numpy()[bt, 0]
    moved = fused[a.bt]
    assert np.array_equal(b.scale_k[moved], a.scale_k[moved] * fkx[moved])
    assert np.array_equal(b.scale_v[moved], a.scale_v[moved] * fvx[moved])
    assert (a.scale_k[~moved] == 1.0).all() and (b.scale_k[~moved] == 1.0).all()      # untouched blocks stay raw


def test_threshold_above_one_changes_nothing(oracle):
    rec = wl.tiny_bff()
    m = wl.materialise(rec, "cpu")
    for g in range(rec.G):
        K, V = m["K"][g].numpy(), m["V"][g].numpy()
        res = oracle.fuse_group(K, V, m["bt"][g].numpy(), rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, thr=1.5)
        assert np.array_equal(res.bt, np.arange(rec.n)) and np.array_equal(res.kpool, K) and np.array_equal(res.vpool, V)
        assert (res.scale_k == 1.0).all() and (res.scale_v == 1.0).all() and (res.refcount == 1).all()
        assert res.compression_ratio == 1.0 and len(res.free_list) == 0


def test_tiny_config_planted_pairs_give_22_physical_blocks(oracle):
    """Config 1: ten disjoint cross-request pairs, random cosines ~ N(0, 1/1024) far below 0.95."""
    rec = wl.tiny_bff()
    assert len(rec.notes["pairs"]) == 10
    m = wl.materialise(rec, "cpu")
    for g in range(rec.G):
        res = oracle.fuse_group(m["K"][g].numpy(), m["V"][g].numpy(), m["bt"][g].numpy(), rec.leaf_start,
                                rec.leaf_count, rec.unit_leaf_ptr, thr=rec.thr)
        assert res.n_physical == 22
        assert math.isclose(res.compression_ratio, 32 / 22)
        for a, b in rec.notes["pairs"]:
            assert res.bt[a] == res.bt[b] == min(a, b)       # the copy in the later request points at the earlier one
        assert res.stats[1] == 10 and res.stats[2] == 0       # 10 fused, none within 1e-3 of the threshold


def test_planted_cosines_follow_closed_form(oracle):
    """base vs noisy copy ~ 1/sqrt(1+s^2); copy vs copy ~ 1/(1+s^2) for large r."""
    rng = np.random.default_rng(7)
    r, s = 4096, 0.3
    base = rng.standard_normal(r)
    K = np.stack([base, base + s * rng.standard_normal(r), base + s * rng.standard_normal(r)]).astype(np.float32)
    nrm = oracle.block_norms(K)
    S = oracle.similarity(K, nrm, np.array([0, 1]), np.array([1, 2]))
    assert abs(S[0, 0] - 1 / math.sqrt(1 + s * s)) < 0.01
    assert abs(S[1, 1] - 1 / (1 + s * s)) < 0.015
    assert abs(S[1, 0] - 1.0) < 1e-12


# ---------------------------------------------------------------- independent dense brute force

def _round_store(x64, kind):
    if kind == "f32":
        return x64.astype(np.float32)
    # bfloat16: choose between the two neighbouring grid points by exact distance, ties to even mantissa
    f = x64.astype(np.float32)
    b = f.view(np.uint32)
    lo = (b & np.uint32(0xFFFF0000))
    hi = lo + np.uint32(0x10000)
    lo64 = lo.view(np.float32).astype(np.float64)
    hi64 = hi.view(np.float32).astype(np.float64)
    dl, dh = np.abs(x64 - lo64), np.abs(hi64 - x64)
    pick_hi = (dh < dl) | ((dh == dl) & ((lo >> 16) & 1 == 1))
    return (np.where(pick_hi, hi, lo) >> 16).astype(np.uint16)


def _widen(p):
    return wl_to_f64(p) if p.dtype == np.uint16 else p.astype(np.float64)


def _brute_force(K, V, bt, leaves_of_units, thr, kind, rule="argmax"):
    """Dense, list-based restatement of Algorithm 1 written independently of the C oracle."""
    K, V, bt = K.copy(), V.copy(), bt.copy()
    n = len(bt)
    orig_k = np.linalg.norm(_widen(K), axis=1)[bt]
    orig_v = np.linalg.norm(_widen(V), axis=1)[bt]
    freed = []

    def node(Ls, Rs):
        if not Ls or not Rs:
            return Ls + Rs
        kl, kr = _widen(K[Ls]), _widen(K[Rs])
        nl, nr = np.linalg.norm(kl, axis=1), np.linalg.norm(kr, axis=1)
        sim = (kl @ kr.T) / np.outer(np.where(nl == 0, np.inf, nl), np.where(nr == 0, np.inf, nr))
        tgt = {}
        for j in range(len(Rs)):
            if rule == "first_row":                 # lowest row above the threshold
                above = np.nonzero(sim[:, j] > thr)[0]
                if len(above):
                    tgt.setdefault(int(above[0]), []).append(j)
                continue
            i = int(np.argmax(sim[:, j]))           # numpy argmax: first maximum
            if sim[i, j] > thr:
                tgt.setdefault(i, []).append(j)
        for pool in (K, V):
            for i, js in tgt.items():
                w = _widen(pool[[Ls[i]] + [Rs[j] for j in js]])
                nn = np.linalg.norm(w, axis=1, keepdims=True)
                s = (w / np.where(nn == 0, np.inf, nn)).sum(0)
                ln = np.linalg.norm(s)
                pool[Ls[i]] = _round_store(s / ln if ln > 0 else s, kind)
        gone = set()
        for i, js in tgt.items():
            for j in js:
                bt[bt == Rs[j]] = Ls[i]
                freed.append(Rs[j])
                gone.add(j)
        return Ls + [Rs[j] for j in range(len(Rs)) if j not in gone]

    def ff(sets):
        if len(sets) == 1:
            return sets[0]
        h = len(sets) // 2
        return node(ff(sets[:h]), ff(sets[h:]))

    def ff_unit(unit_leaves):
        return ff([list(bt[s:s + c]) for s, c in unit_leaves]) if unit_leaves else []

    def ff_units(units):
        if len(units) == 1:
            return ff_unit(units[0])
        h = len(units) // 2
        return node(ff_units(units[:h]), ff_units(units[h:]))

    ff_units(leaves_of_units)
    nk, nv = np.linalg.norm(_widen(K), axis=1), np.linalg.norm(_widen(V), axis=1)
    safe = lambda o, c: np.where(c == 0, 1.0, o / np.where(c == 0, 1.0, c))     # an untouched zero block keeps scale 1
    return K, V, bt, safe(orig_k, nk[bt]), safe(orig_v, nv[bt]), sorted(freed)


@pytest.mark.parametrize("rule", ["argmax", "first_row"])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("leaves", [[5, 3, 4, 6, 2], [4, 4, 4, 4], [7, 1, 1, 6, 3, 2, 5]])
def test_oracle_equals_dense_brute_force(oracle, kind, leaves, rule):
    rng = np.random.default_rng(sum(leaves) + len(kind))
    n, r = sum(leaves), 40
    protos = rng.standard_normal((6, r))
    pick = rng.integers(0, 6, size=n)
    X = np.where(rng.random(n)[:, None] < 0.7, protos[pick] + 0.15 * rng.standard_normal((n, r)), rng.standard_normal((n, r)))
    Y = np.where(rng.random(n)[:, None] < 0.7, protos[pick][:, ::-1] + 0.15 * rng.standard_normal((n, r)), rng.standard_normal((n, r)))
    X[3] = 0.0                                   # a zero block never fuses
    if kind == "f32":
        K, V = X.astype(np.float32), Y.astype(np.float32)
    else:
        K, V = _bf16_bits(X), _bf16_bits(Y)
    perm = rng.permutation(n).astype(np.int32)   # paged layout: logical x lives at physical perm[x]
    Kp, Vp = np.empty_like(K), np.empty_like(V)
    Kp[perm], Vp[perm] = K, V
    lc = np.asarray(leaves, np.int32)
    ls = np.concatenate([[0], np.cumsum(lc)[:-1]]).astype(np.int32)
    up = np.arange(len(leaves) + 1, dtype=np.int32)
    thr = 0.8
    res = oracle.fuse_group(Kp, Vp, perm, ls, lc, up, thr=thr, rule=rule)
    bK, bV, bbt, bsk, bsv, bfreed = _brute_force(Kp, Vp, perm, [[(int(s), int(c))] for s, c in zip(ls, lc)], thr, kind, rule)
    assert res.stats[1] >= 3, "test input should actually fuse something"
    assert np.array_equal(res.bt, bbt)
    assert np.array_equal(res.kpool, bK) and np.array_equal(res.vpool, bV)
    assert np.allclose(res.scale_k, bsk, rtol=1e-12) and np.allclose(res.scale_v, bsv, rtol=1e-12)
    assert sorted(res.free_list.tolist()) == bfreed
    # conservation: every logical block counted once, freed + live = used, nothing points at a freed block
    assert res.refcount.sum() == n
    assert len(set(res.bt.tolist())) + len(res.free_list) == n
    assert not set(res.bt.tolist()) & set(res.free_list.tolist())
    assert len(set(res.free_list.tolist())) == len(res.free_list)
    assert np.array_equal(np.bincount(res.bt, minlength=n), res.refcount)
    # fused representatives are unit vectors up to storage rounding
    live_fused = [p for p in set(res.bt.tolist()) if res.refcount[p] > 1]
    tol = 2e-7 if kind == "f32" else 3e-3
    assert all(abs(res.norm_k[p] - 1.0) < tol for p in live_fused)


def test_chunks_then_requests_and_group_size(oracle):
    """Units with several leaves fuse their chunks first; group_size cuts the unit list into independent trees."""
    rng = np.random.default_rng(11)
    r = 32
    units = [[3, 2], [4], [2, 2, 1], [3]]
    n = sum(sum(u) for u in units)
    protos = rng.standard_normal((4, r))
    K = (protos[rng.integers(0, 4, n)] + 0.1 * rng.standard_normal((n, r))).astype(np.float32)
    V = rng.standard_normal((n, r)).astype(np.float32)
    bt = np.arange(n, dtype=np.int32)
    lc = np.asarray([c for u in units for c in u], np.int32)
    ls = np.concatenate([[0], np.cumsum(lc)[:-1]]).astype(np.int32)
    up = np.concatenate([[0], np.cumsum([len(u) for u in units])]).astype(np.int32)
    res = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.85)
    spec = []
    k = 0
    for u in units:
        spec.append([(int(ls[k + i]), int(lc[k + i])) for i in range(len(u))])
        k += len(u)
    bK, bV, bbt, *_ = _brute_force(K, V, bt, spec, 0.85, "f32")
    assert np.array_equal(res.bt, bbt) and np.array_equal(res.kpool, bK) and np.array_equal(res.vpool, bV)
    # group_size 2: units {0,1} and {2,3} never meet -> equals two separate runs
    res2 = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.85, group_size=2)
    b2K, b2V, b2bt, *_ = _brute_force(K, V, bt, spec[:2], 0.85, "f32")
    b3K, b3V, b3bt, *_ = _brute_force(b2K, b2V, b2bt, spec[2:], 0.85, "f32")
    assert np.array_equal(res2.bt, b3bt) and np.array_equal(res2.kpool, b3K)
    first_half = set(range(int(ls[up[2]])))
    assert all((res2.bt[x] in first_half) == (x in first_half) for x in range(n))


def test_sharing_the_columns_of_a_node_over_threads_changes_nothing(oracle):
    """The oracle may spread the independent columns of a node over host threads (for the groups of tens of thousands
    of blocks); tables, pools, scales, statistics and the decision trace must not depend on the thread count."""
    rec = wl.zipf_bff(n_req=8, tokens=32 * 24, layers=1, kv_heads=1, pool=120)
    mat = wl.materialise(rec, "cpu")
    K, V, bt = wl.to_numpy_pool(mat["K"][0]), wl.to_numpy_pool(mat["V"][0]), mat["bt"][0].numpy().copy()
    runs = []
    try:
        for threads in (1, 4):
            oracle.set_column_threads(threads)
            runs.append(oracle.fuse_group(K, V, bt, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr, want_trace=True))
    finally:
        oracle.set_column_threads(1)
    a, b = runs
    assert a.stats[1] > 0
    for field in ("bt", "kpool", "vpool", "refcount", "scale_k", "scale_v", "norm_k", "norm_v", "stats", "free_list", "trace"):
        assert np.array_equal(getattr(a, field), getattr(b, field)), field


def test_groups_are_independent_and_deterministic(oracle):
    rec = wl.llama8b_bff(n_req=4, tokens=256, layers=1, kv_heads=3, prefix_tokens=64, near_pool=8, d=32)
    m = wl.materialise(rec, "cpu")
    Ks = [wl.to_numpy_pool(m["K"][g]) for g in range(3)]
    Vs = [wl.to_numpy_pool(m["V"][g]) for g in range(3)]
    bts = [m["bt"][g].numpy() for g in range(3)]
    a = oracle.fuse_groups(Ks, Vs, bts, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr, threads=3)
    b = oracle.fuse_groups(Ks[::-1], Vs[::-1], bts[::-1], rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, rec.thr)[::-1]
    for x, y in zip(a, b):
        assert np.array_equal(x.bt, y.bt) and np.array_equal(x.kpool, y.kpool) and np.array_equal(x.scale_v, y.scale_v)
    # the shared prefix (4 blocks) collapses across the 4 requests in every group
    p = rec.req_blocks[0]
    for x in a:
        for blk in range(4):
            assert len({int(x.bt[q * p + blk]) for q in range(4)}) == 1


# ---------------------------------------------------------------- decode attention

def _textbook_attention(q, Ktok, Vtok, sm):
    z = sm * (Ktok @ q)
    w = np.exp(z - z.max())
    return (w / w.sum()) @ Vtok


def test_attention_reduces_to_textbook_softmax_when_nothing_is_fused(oracle):
    rng = np.random.default_rng(13)
    H, Hq, t, d, B = 2, 4, 4, 8, 3
    ctx = np.array([10, 16, 1], np.int32)                 # partial tail, full, single token
    blocks = (ctx + t - 1) // t
    n = int(blocks.sum())
    req_start = np.concatenate([[0], np.cumsum(blocks)[:-1]]).astype(np.int32)
    K = rng.standard_normal((H, n, t * d)).astype(np.float32)
    V = rng.standard_normal((H, n, t * d)).astype(np.float32)
    perm = np.stack([rng.permutation(n) for _ in range(H)]).astype(np.int32)
    Kp, Vp = np.empty_like(K), np.empty_like(V)
    for g in range(H):
        Kp[g][perm[g]] = K[g]
        Vp[g][perm[g]] = V[g]
    q = rng.standard_normal((B, Hq, d))
    one = np.ones((H, n))
    out = oracle.paged_decode_attention(q, Kp, Vp, perm, one, one, req_start, ctx, t, d)
    for b in range(B):
        for h in range(Hq):
            g = h // (Hq // H)
            kt = K[g][req_start[b]: req_start[b] + blocks[b]].reshape(-1, d)[: ctx[b]].astype(np.float64)
            vt = V[g][req_start[b]: req_start[b] + blocks[b]].reshape(-1, d)[: ctx[b]].astype(np.float64)
            assert np.allclose(out[b, h], _textbook_attention(q[b, h], kt, vt, 1 / math.sqrt(d)), atol=1e-13)
    assert np.allclose(out[2, 0], V[0][req_start[2]].reshape(t, d)[0], atol=1e-13)   # one token: output is its value
    out0 = oracle.paged_decode_attention(np.zeros_like(q), Kp, Vp, perm, one, one, req_start, ctx, t, d)
    assert np.allclose(out0[1, 3], V[1][req_start[1]: req_start[1] + 4].reshape(-1, d).mean(0), atol=1e-13)  # q = 0: mean value


def test_attention_uses_per_logical_block_scales(oracle):
    """Two logical blocks sharing one stored unit block with scales a, b must equal attention over a*block and b*block."""
    rng = np.random.default_rng(17)
    t, d = 4, 8
    blk_k = rng.standard_normal(t * d)
    blk_v = rng.standard_normal(t * d)
    K = blk_k[None, None, :].astype(np.float32)
    V = blk_v[None, None, :].astype(np.float32)
    bt = np.array([[0, 0]], np.int32)
    sk, sv = np.array([[0.5, 3.0]]), np.array([[2.0, 0.25]])
    q = rng.standard_normal((1, 1, d))
    out = oracle.paged_decode_attention(q, K, V, bt, sk, sv, np.array([0]), np.array([2 * t]), t, d)
    k32, v32 = K[0, 0].astype(np.float64).reshape(t, d), V[0, 0].astype(np.float64).reshape(t, d)
    kt = np.concatenate([0.5 * k32, 3.0 * k32])
    vt = np.concatenate([2.0 * v32, 0.25 * v32])
    assert np.allclose(out[0, 0], _textbook_attention(q[0, 0], kt, vt, 1 / math.sqrt(d)), atol=1e-13)


def test_fusion_then_attention_satisfies_softmax_drift_bound(oracle):
    """Appendix proof: ||s' - s||_1 <= exp(2 eps) - 1 with eps = max |logit change|."""
    rec = wl.tiny_bff()
    m = wl.materialise(rec, "cpu")
    g = 0
    K, V, bt = m["K"][g].numpy(), m["V"][g].numpy(), m["bt"][g].numpy()
    res = oracle.fuse_group(K, V, bt, rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, thr=rec.thr)
    q = np.random.default_rng(19).standard_normal(rec.d)
    sm = 1 / math.sqrt(rec.d)
    b = 1
    xs = np.arange(rec.req_start[b], rec.req_start[b] + rec.req_blocks[b])
    z0 = sm * (K[bt[xs]].astype(np.float64).reshape(-1, rec.d) @ q)
    z1 = sm * ((res.kpool[res.bt[xs]].astype(np.float64) * res.scale_k[xs, None]).reshape(-1, rec.d) @ q)
    s0 = np.exp(z0 - z0.max()); s0 /= s0.sum()
    s1 = np.exp(z1 - z1.max()); s1 /= s1.sum()
    eps = np.abs(z1 - z0).max()
    assert eps > 0 and np.abs(s1 - s0).sum() <= math.exp(2 * eps) - 1 + 1e-12


# ---------------------------------------------------------------- variants: row-order rule, request order, evaluation modes

def test_first_row_rule_hand_example_and_relation_to_argmax(oracle):
    """Algorithm 1's loop over the rows of sim taken literally: a row takes every block above thr that is still
    there.  Column 0: rows 0 (0.9) and 1 (0.95) both clear 0.7 -> row 0 was first; the arg-max reading gives row 1."""
    S = np.array([[0.90, 0.20, 0.95, 0.70],
                  [0.95, 0.80, 0.10, 0.70],
                  [0.10, 0.85, 0.97, 0.6999]])
    assert oracle.assign_first_row(S, 0.7).tolist() == [0, 1, 0, -1]     # 0.7 > 0.7 is false
    assert oracle.assign(S, 0.7)[0].tolist() == [1, 2, 2, -1]
    assert oracle.assign_first_row(S, 1.5).tolist() == [-1, -1, -1, -1]
    rng = np.random.default_rng(23)
    for _ in range(50):
        ml, mr = rng.integers(1, 9), rng.integers(1, 9)
        S = rng.random((ml, mr))
        u = float(rng.uniform(0.3, 0.95))
        a1 = oracle.assign_first_row(S, u)
        a0 = oracle.assign(S, u)[0]
        above = S > u
        want = np.where(above.any(0), above.argmax(0), -1)               # first True per column
        assert a1.tolist() == want.tolist()
        assert ((a1 >= 0) == (a0 >= 0)).all()                            # the same blocks fuse, maybe elsewhere
        single = above.sum(0) <= 1
        assert (a1[single] == a0[single]).all()                          # the readings differ only on contested blocks


def test_first_row_rule_changes_contested_blocks_only(oracle):
    """Left leaf {a, a'} with a' a near copy of a, right leaf {b} nearest to a': arg-max sends b to a', the row
    loop to a (the first row above the threshold)."""
    e = np.eye(4)
    a, a2, b = e[0], e[0] + 0.10 * e[1], e[0] + 0.12 * e[1]
    K = np.stack([a, a2, b]).astype(np.float32)
    V = np.stack([e[2], e[3], e[2] + e[3]]).astype(np.float32)
    bt, ls, lc, up = _identity_setup(K, V, [2, 1])
    r0 = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.9)
    r1 = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.9, rule="first_row")
    assert r0.bt.tolist() == [0, 1, 1] and r1.bt.tolist() == [0, 1, 0]
    assert r0.n_physical == r1.n_physical == 2
    assert np.array_equal(r1.kpool[1], K[1]) and not np.array_equal(r1.kpool[0], K[0])


def test_shortest_first_order_and_the_remark_best_case(oracle):
    """Remark after Algorithm 1: shorter requests on the left; in the best case every block of the right tree
    is unified into the left tree.  Short request {x, y}, long request {x, y, x, y, x, y}: blocks of one request
    are never compared with each other, so long-first keeps all six blocks of the long request, short-first
    keeps two."""
    ls, lc, up, order = oracle.shortest_first([0, 5, 8, 12], [5, 3, 4, 3], [0, 1, 2, 3, 4])
    assert order.tolist() == [1, 3, 2, 0] and ls.tolist() == [5, 12, 8, 0] and lc.tolist() == [3, 3, 4, 5]
    assert up.tolist() == [0, 1, 2, 3, 4]
    # units with several leaves move as a whole and keep their chunk order
    ls, lc, up, order = oracle.shortest_first([0, 4, 8, 10], [4, 4, 2, 3], [0, 2, 3, 4])
    assert order.tolist() == [1, 2, 0] and ls.tolist() == [8, 10, 0, 4] and lc.tolist() == [2, 3, 4, 4]
    assert up.tolist() == [0, 1, 2, 4]
    # one unit: its leaves are ordered
    ls, lc, up, order = oracle.shortest_first([0, 4, 8], [4, 4, 1], [0, 3])
    assert order.tolist() == [2, 0, 1] and ls.tolist() == [8, 0, 4] and up.tolist() == [0, 3]

    rng = np.random.default_rng(29)
    x, y = rng.standard_normal(16), rng.standard_normal(16)
    K = np.stack([x, y, x, y, x, y, x, y]).astype(np.float32)       # long request first in the table, then the short one
    K *= rng.uniform(0.5, 2.0, size=(8, 1)).astype(np.float32)      # same directions, different norms
    V = rng.standard_normal((8, 16)).astype(np.float32)
    bt = np.arange(8, dtype=np.int32)
    given = ([0, 6], [6, 2], [0, 1, 2])
    long_first = oracle.fuse_group(K, V, bt, *given, thr=0.99)
    ls, lc, up, order = oracle.shortest_first(*given)
    assert order.tolist() == [1, 0] and ls.tolist() == [6, 0]
    short_first = oracle.fuse_group(K, V, bt, ls, lc, up, thr=0.99)
    assert long_first.n_physical == 6 and short_first.n_physical == 2
    assert short_first.compression_ratio == 4.0
    assert set(short_first.bt.tolist()) == {6, 7}                   # everything points into the short request's blocks
    assert np.allclose(short_first.scale_k * short_first.norm_k[short_first.bt], np.linalg.norm(K.astype(np.float64), axis=1), rtol=1e-6)


@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_replicate_rescaled_closed_form_and_attention_equivalence(oracle, kind):
    """First evaluation mode of the results section: every logical block gets its own block back, holding
    scale * representative."""
    # closed form (two-block bisector case): rep = (2, 1)/sqrt5, scales 1 and 2.5
    K = np.array([[1.0, 0.0], [1.5, 2.0]], np.float32)
    V = np.array([[0.0, 3.0], [4.0, 0.0]], np.float32)
    bt0, ls, lc, up = _identity_setup(K, V, [1, 1])
    res = oracle.fuse_group(K, V, bt0, ls, lc, up, thr=0.5)
    Kr = oracle.replicate_rescaled(res.kpool, bt0, res.bt, res.scale_k)
    Vr = oracle.replicate_rescaled(res.vpool, bt0, res.bt, res.scale_v)
    assert np.allclose(Kr, [[2 / math.sqrt(5), 1 / math.sqrt(5)], [5 / math.sqrt(5), 2.5 / math.sqrt(5)]], rtol=3e-7)
    assert np.allclose(Vr, [[3 / math.sqrt(2), 3 / math.sqrt(2)], [4 / math.sqrt(2), 4 / math.sqrt(2)]], rtol=3e-7)

    # a fused workload: attention over the replicated cache with the original table and no scales equals
    # attention through the fused table, up to the rounding of scale * representative into the pool type
    rec = wl.llama8b_bff(n_req=4, tokens=256, layers=1, kv_heads=2, prefix_tokens=64, near_pool=8, d=32,
                         dtype=torch.float32 if kind == "f32" else torch.bfloat16)
    m = wl.materialise(rec, "cpu", phys_perm=True)
    H = rec.G
    Ks = [wl.to_numpy_pool(m["K"][g]) for g in range(H)]
    Vs = [wl.to_numpy_pool(m["V"][g]) for g in range(H)]
    bts = [m["bt"][g].numpy().copy() for g in range(H)]
    res = [oracle.fuse_group(Ks[g], Vs[g], bts[g], rec.leaf_start, rec.leaf_count, rec.unit_leaf_ptr, thr=rec.thr) for g in range(H)]
    assert sum(int(r.stats[1]) for r in res) > 20
    Kr = [oracle.replicate_rescaled(res[g].kpool, bts[g], res[g].bt, res[g].scale_k) for g in range(H)]
    Vr = [oracle.replicate_rescaled(res[g].vpool, bts[g], res[g].bt, res[g].scale_v) for g in range(H)]
    for g in range(H):
        untouched = [x for x in range(rec.n) if res[g].bt[x] == bts[g][x] and res[g].scale_k[x] == 1.0]
        assert len(untouched) > 10
        assert all(np.array_equal(Kr[g][bts[g][x]], Ks[g][bts[g][x]]) for x in untouched)   # never-fused blocks: byte for byte
        # every element is the storage value nearest to the product, by the test's own rounding
        x = next(x for x in range(rec.n) if res[g].bt[x] != bts[g][x])
        prod = float(np.float32(res[g].scale_k[x])) * oracle.pool_to_f64(res[g].kpool[res[g].bt[x]])
        assert np.array_equal(Kr[g][bts[g][x]], _round_store(prod, kind))
    q = np.random.default_rng(31).standard_normal((rec.B, 4, rec.d))
    one = np.ones((H, rec.n))
    fused = oracle.paged_decode_attention(q, [r.kpool for r in res], [r.vpool for r in res], [r.bt for r in res],
                                          [r.scale_k for r in res], [r.scale_v for r in res], rec.req_start, rec.ctx_len, rec.t, rec.d)
    repl = oracle.paged_decode_attention(q, Kr, Vr, bts, one, one, rec.req_start, rec.ctx_len, rec.t, rec.d)
    tol = 2e-6 if kind == "f32" else 2e-2
    assert np.abs(fused - repl).max() <= tol * np.abs(fused).max()
    assert np.abs(fused - repl).max() > 0


# ---------------------------------------------------------------- threshold control statistics (analysis section)

def test_exceedance_rate_closed_forms_and_inverse():
    from oracle import threshold as th
    n, mu, sigma = 5000.0, 0.2, 0.1
    assert th.exceedance_rate(n, mu, sigma, mu) == pytest.approx(n / 2, rel=1e-15)
    # 1 - Phi(1), 1 - Phi(2), 1 - Phi(3): textbook values of the normal tail
    for k, tail in ((1, 0.15865525393145707), (2, 0.022750131948179195), (3, 0.0013498980316300933)):
        assert th.exceedance_rate(n, mu, sigma, mu + k * sigma) == pytest.approx(n * tail, rel=1e-12)
        assert th.exceedance_rate(n, mu, sigma, mu - k * sigma) == pytest.approx(n * (1 - tail), rel=1e-12)
    for u in (0.25, 0.4, 0.55):
        lam = th.exceedance_rate(n, mu, sigma, u)
        assert th.threshold_for_rate(n, mu, sigma, lam) == pytest.approx(u, abs=1e-10)
    # degenerate spread: everything or nothing exceeds
    assert th.exceedance_rate(n, 0.5, 0.0, 0.4) == n and th.exceedance_rate(n, 0.3, 0.0, 0.4) == 0.0


def test_exceedance_rate_predicts_gaussian_counts():
    from oracle import threshold as th
    rng = np.random.default_rng(11)
    x = rng.normal(0.3, 0.07, 200_000)
    mu, var = th.moments(x)
    assert mu == pytest.approx(x.mean(), rel=1e-12) and var == pytest.approx(x.var(), rel=1e-10)
    for u in (0.45, 0.5, 0.55):
        lam = th.exceedance_rate(len(x), mu, math.sqrt(var), u)
        cnt = int((x > u).sum())
        assert abs(cnt - lam) <= 4 * math.sqrt(lam) + 0.02 * lam


def test_compression_corollary_closed_forms():
    from oracle import threshold as th
    cr, p0 = th.predicted_compression([10.0, 30.0], 100.0)        # 200 blocks, 40 expected fusions
    assert cr == pytest.approx(200.0 / 160.0, rel=1e-15)
    assert p0[0] == pytest.approx(math.exp(-10.0)) and p0[1] == pytest.approx(math.exp(-30.0))
    cr, p0 = th.predicted_compression([math.log(2.0)], 50.0)
    assert p0[0] == pytest.approx(0.5, rel=1e-15)
    cr, p0 = th.predicted_compression([0.0, 0.0, 0.0], 64.0)
    assert cr == 1.0 and (p0 == 1.0).all()


def test_pair_cosines_and_feedback_direction():
    from oracle import threshold as th
    K = np.array([[1.0, 0.0], [1.2, 1.6], [0.0, 3.0], [0.0, 0.0], [2.0, 0.0]])
    bt = np.array([4, 1, 2, 3, 0])             # logical -> physical
    cos = th.pair_cosines(K, bt, np.array([[0, 1], [0, 2], [1, 2], [0, 4], [3, 1]]))
    assert cos == pytest.approx([0.6, 0.0, 0.8, 1.0, 0.0], abs=1e-15)
    assert th.feedback_step(0.9, 2.0, 1.5, 0.1, 0.5, 0.99) > 0.9       # too much compression: raise
    assert th.feedback_step(0.9, 1.1, 1.5, 0.1, 0.5, 0.99) < 0.9       # too little: lower
    assert th.feedback_step(0.9, 1.5, 1.5, 0.1, 0.5, 0.99) == 0.9
    assert th.feedback_step(0.98, 9.0, 1.5, 0.5, 0.5, 0.99) == 0.99    # clamped


# ---------------------------------------------------------------- causal prefill attention through the table

def test_causal_prefill_attention_equals_library_causal_attention_and_decode(oracle):
    """Nothing fused: the oracle must equal a library causal attention (torch SDPA with a causal mask, fp64);
    with a fused table, the row of the query at position pos must equal the decode oracle with ctx_len = pos + 1."""
    rng = np.random.default_rng(21)
    H, Hq, t, d, N = 2, 4, 4, 8, 37
    nb = (N + t - 1) // t
    n = nb + 3
    req_start = 2
    K = rng.standard_normal((H, n, t * d)).astype(np.float32)
    V = rng.standard_normal((H, n, t * d)).astype(np.float32)
    bt = np.stack([rng.permutation(n) for _ in range(H)]).astype(np.int32)
    one = np.ones((H, n))
    q = rng.standard_normal((N, Hq, d))
    out = oracle.causal_prefill_attention(q, np.arange(N), K, V, bt, one, one, req_start, t, d)
    for h in range(Hq):
        g = h // (Hq // H)
        xs = bt[g][req_start: req_start + nb]
        kt = torch.tensor(K[g][xs].reshape(-1, d)[:N], dtype=torch.float64)
        vt = torch.tensor(V[g][xs].reshape(-1, d)[:N], dtype=torch.float64)
        ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(q[:, h])[None], kt[None], vt[None], is_causal=True)[0]
        assert np.allclose(out[:, h], ref.numpy(), atol=1e-12)
    assert np.allclose(out[0, 0], V[0][bt[0][req_start]].reshape(t, d)[0], atol=1e-13)   # first token sees only itself
    # fused table: two logical blocks share a stored block with different scales
    bt2 = bt.copy()
    bt2[:, req_start + 5] = bt2[:, req_start + 1]
    sk, sv = rng.uniform(0.5, 2.0, (H, n)), rng.uniform(0.5, 2.0, (H, n))
    pos = np.array([3, 22, 23, 36])
    out2 = oracle.causal_prefill_attention(q[pos], pos, K, V, bt2, sk, sv, req_start, t, d)
    for i, p in enumerate(pos):
        dec = oracle.paged_decode_attention(q[p][None], K, V, bt2, sk, sv, np.array([req_start]), np.array([p + 1]), t, d)
        assert np.allclose(out2[i], dec[0], atol=1e-13)
