"""CPU checks of the two inequalities the opt-in screens of the similarity step rest on (no GPU, no library code):

* prefix screen:  cos(a, b) <= <a[:p], b[:p]> / (|a| |b|) + tail(a) tail(b),  tail(x) = |x[p:]| / |x|
* fp8 screen:     |cos(a, b) - <q(a), q(b)> / S^2| <= err(a) + err(b) + err(a) err(b),
                  q(x) = nearest e4m3 value of every element of S x / |x|,  err(x) = |x / |x| - q(x) / S|
* centred copies: with m any binary32 vector of norm 1 to rounding, alpha = <m, u> rounded to binary32, u_c = u - alpha m,
                  c any estimate of |u_c| within a factor 1.15, q = e4m3(u_c S / c), s = binary32(c / S):
                  |cos(a, b) - (<q(a), q(b)> s_a s_b + alpha_a alpha_b)| <= e_a + e_b + e_a e_b,
                  e = |u_c - q s| + 2e-6  (the margin covers the roundings of m and alpha)

The e4m3 values are written out from the format's definition (4 exponent bits, bias 7, 3 mantissa bits, subnormals,
largest finite value 448) and rounding is done by a nearest-value search, independently of any conversion routine.  The
inputs include the cases where the bounds are tight or the copies are bad: parallel vectors, vectors whose energy sits
in the tail or in one element, values that underflow the format."""
import numpy as np
import pytest

S = 256.0


def _e4m3_values():
    vals = []
    for e in range(16):
        for m in range(8):
            if e == 15 and m == 7:
                continue                      # NaN
            vals.append(m / 8.0 * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    v = np.array(sorted(set(vals)))
    return np.concatenate([-v[::-1], v])


def _nearest(table, x):
    idx = np.searchsorted(table, x).clip(1, len(table) - 1)
    lo, hi = table[idx - 1], table[idx]
    return np.where(np.abs(x - lo) <= np.abs(hi - x), lo, hi)


def _cases(rng, r):
    a = rng.standard_normal(r)
    yield "unrelated", a, rng.standard_normal(r)
    yield "parallel", a, 3.5 * a
    yield "opposite", a, -a
    yield "near copy", a, a + 0.05 * rng.standard_normal(r)
    spike = np.full(r, 1e-4)
    spike[r - 1] = 50.0
    yield "energy in the last element", spike, spike + 1e-5 * rng.standard_normal(r)
    yield "one spike against noise", spike, rng.standard_normal(r)
    tiny = 1e-30 * rng.standard_normal(r)
    yield "tiny values", tiny, tiny + 1e-31 * rng.standard_normal(r)
    head = np.concatenate([rng.standard_normal(r // 4), np.zeros(r - r // 4)])
    yield "energy in the head only", head, head + 0.01 * rng.standard_normal(r)


@pytest.mark.parametrize("r", [128, 2048])
def test_prefix_bound_holds(r):
    rng = np.random.default_rng(7 + r)
    for name, a, b in _cases(rng, r):
        na, nb = np.linalg.norm(a), np.linalg.norm(b)
        cos = float(a @ b) / (na * nb)
        for p in (64, r // 4, r // 2, r - 64):
            head = float(a[:p] @ b[:p]) / (na * nb)
            bound = head + np.linalg.norm(a[p:]) / na * np.linalg.norm(b[p:]) / nb
            assert cos <= bound + 1e-12, (name, p)
        # tight for parallel vectors: the bound is the cosine itself
        if name == "parallel":
            assert abs(bound - 1.0) < 1e-12


@pytest.mark.parametrize("r", [128, 2048])
def test_fp8_copy_bound_holds_and_is_small_on_noise(r):
    table = _e4m3_values()
    assert table.max() == 448.0 and len(table) == 2 * 127        # 126 positive values and a zero, mirrored
    rng = np.random.default_rng(11 + r)
    for name, a, b in _cases(rng, r):
        u, v = a / np.linalg.norm(a), b / np.linalg.norm(b)
        qu, qv = _nearest(table, S * u), _nearest(table, S * v)
        eu, ev = np.linalg.norm(u - qu / S), np.linalg.norm(v - qv / S)
        cos, cos_q = float(u @ v), float(qu @ qv) / (S * S)
        assert abs(cos - cos_q) <= eu + ev + eu * ev + 1e-12, name
        if name in ("unrelated", "near copy", "parallel"):
            assert eu < 0.04 and ev < 0.04, name                       # 3 mantissa bits: about 0.027 on noise
    # identical blocks have identical copies: their product is the same whichever is left or right
    a = rng.standard_normal(r)
    q = _nearest(table, S * a / np.linalg.norm(a))
    assert float(q @ q) / (S * S) == pytest.approx(1.0, abs=0.06)


@pytest.mark.parametrize("r", [128, 2048])
@pytest.mark.parametrize("direction", ["mean of the blocks", "unrelated to the blocks", "one of the blocks"])
def test_centred_fp8_copy_bound_holds_for_any_direction(r, direction):
    """The screen stays exact whatever direction is taken out; a direction the blocks share makes the bound small."""
    table = _e4m3_values()
    rng = np.random.default_rng(23 + r)
    common = 2.0 * rng.standard_normal(r)
    blocks = [common + rng.standard_normal(r) for _ in range(12)]
    blocks += [blocks[0].copy(), blocks[1] + 0.05 * rng.standard_normal(r), 3.0 * blocks[2], -blocks[3],
               rng.standard_normal(r), common.copy(), 1e-30 * blocks[4]]
    units = [b / np.linalg.norm(b) for b in blocks]
    if direction == "mean of the blocks":
        m64 = np.sum(units[:8], axis=0)
    elif direction == "unrelated to the blocks":
        m64 = rng.standard_normal(r)
    else:
        m64 = units[5].copy()
    m = (m64 / np.linalg.norm(m64)).astype(np.float32).astype(np.float64)       # stored as binary32: not exactly unit
    assert abs(m @ m - 1.0) < 2.0 ** -22

    def copy_of(u, gain_error):
        alpha = float(np.float32(m @ u))
        uc = u - alpha * m
        c = max(np.sqrt(max(1.0 + alpha * (alpha - 2.0 * (m @ u)), 1e-6)), 1e-3) * gain_error
        s = float(np.float32(c / S))
        target = uc / s
        assert np.abs(target).max() < 448.0                                    # nothing leaves the format's range
        q = _nearest(table, target)
        return q, s, alpha, np.linalg.norm(uc - q * s) + 2e-6, np.linalg.norm(uc)

    copies = [copy_of(u, ge) for u, ge in zip(units, np.resize([1.0, 0.9, 1.15], len(units)))]
    worst, bounds = 0.0, []
    for i, (qa, sa, aa, ea, _) in enumerate(copies):
        for j, (qb, sb, ab, eb, _) in enumerate(copies):
            cos = float(units[i] @ units[j])
            value = float(qa @ qb) * sa * sb + aa * ab
            bound = ea + eb + ea * eb
            assert abs(cos - value) <= bound, (direction, i, j)
            worst = max(worst, abs(cos - value) / bound)
            bounds.append(bound)
    assert worst > 0.01                     # the bound is not vacuous
    if direction == "mean of the blocks":
        # blocks at cosine 0.8 to each other: |u_c| is about 0.45 and the bound shrinks with it (0.054 uncentred)
        assert np.mean([c[4] for c in copies[:12]]) < 0.55 and np.mean(bounds[:12]) < 0.035
    # the block that IS the direction has nothing left to store: zeros (or rounding dust), error at the margin
    if direction == "one of the blocks":
        assert copies[5][3] < 1e-4 and abs(copies[5][2] - 1.0) < 1e-6
