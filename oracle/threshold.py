"""Oracle for the threshold-control statistics -- TEST INFRASTRUCTURE ONLY (see the package docstring).

Analysis section: with the block similarities of a layer approximately Gaussian, mean mu and variance sigma^2 taken
as the sample moments of n similarities, the number of similarities above a threshold u is approximately Poisson
with rate  Lambda(u) = n (1 - Phi((u - mu) / sigma));  the corollary gives the expected compression ratio over L
layers,  L m / (L m - sum_l Lambda_l(u))  with m = m1 + m2 blocks per layer, and the probability that a layer fuses
nothing, exp(-Lambda_l(u)).  The method section's remark on self-adjusting thresholds only fixes the direction of
a feedback step (too much compression -> raise the threshold, and the other way round).

Everything here is the definition written out in fp64 with numpy / math; scipy's erfcinv is the one library
primitive (the inverse of the normal tail).
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erfcinv


def pair_cosines(kpool_f64: np.ndarray, bt: np.ndarray, pairs: np.ndarray) -> np.ndarray:
    """cos(K[bt[i]], K[bt[j]]) for every sampled pair (i, j) of logical blocks of one group; 0 if either is zero."""
    out = np.zeros(len(pairs), np.float64)
    for q, (i, j) in enumerate(np.asarray(pairs)):
        a, b = kpool_f64[bt[i]], kpool_f64[bt[j]]
        na, nb = math.sqrt(float(np.dot(a, a))), math.sqrt(float(np.dot(b, b)))
        out[q] = float(np.dot(a, b)) / (na * nb) if na > 0.0 and nb > 0.0 else 0.0
    return out


def moments(x: np.ndarray):
    """Sample mean and (population) variance, as the analysis section defines mu_l and sigma_l^2."""
    x = np.asarray(x, np.float64)
    mu = float(x.sum() / len(x))
    var = float((x * x).sum() / len(x) - mu * mu)
    return mu, max(var, 0.0)


def exceedance_rate(n: float, mu: float, sigma: float, u: float) -> float:
    """Lambda(u) = n (1 - Phi((u - mu) / sigma))."""
    if sigma <= 0.0:
        return float(n) if mu > u else 0.0
    return float(n) * 0.5 * math.erfc((u - mu) / (sigma * math.sqrt(2.0)))


def threshold_for_rate(n: float, mu: float, sigma: float, rate: float) -> float:
    """The u with Lambda(u) = rate (0 < rate < n)."""
    return mu + sigma * math.sqrt(2.0) * float(erfcinv(2.0 * rate / n))


def predicted_compression(rates, blocks_per_layer: float):
    """Corollary: (compression ratio over the layers, probability of no fusion per layer)."""
    rates = np.asarray(rates, np.float64)
    total = len(rates) * float(blocks_per_layer)
    return total / (total - float(rates.sum())), np.exp(-rates)


def feedback_step(thr: float, observed_cr: float, target_cr: float, gain: float, lo: float, hi: float) -> float:
    """One step of target-compression feedback: compression above the target raises the threshold, below lowers it;
    proportional to the relative miss, clamped to [lo, hi].  Parity unpinned beyond direction and clamp: the paper
    names no gain law, so the proportional form is the builder's own and only its sign and its limits can be held
    against the paper."""
    return min(hi, max(lo, thr + gain * (observed_cr - target_cr) / target_cr))
