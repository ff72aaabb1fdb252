"""CPU checks of the two inequalities the opt-in screens of the similarity step rest on (no GPU, no library code):

* prefix screen:  cos(a, b) <= <a[:p], b[:p]> / (|a| |b|) + tail(a) tail(b),  tail(x) = |x[p:]| / |x|
* fp8 screen:     |cos(a, b) - <q(a), q(b)> / S^2| <= err(a) + err(b) + err(a) err(b),
                  q(x) = nearest e4m3 value of every element of S x / |x|,  err(x) = |x / |x| - q(x) / S|

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
