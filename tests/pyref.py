"""Pure-Python helpers for pinning the oracle: a big-integer Philox4x32-10 and exact rational
probabilities of the stochastic rounding of Eq. (6).  Independent of ``oracle/`` and of the GPU
library; test-only."""
from fractions import Fraction

import numpy as np

_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """Ten rounds on Python integers (arbitrary precision: no overflow behaviour to get wrong)."""
    c = [int(x) & _MASK for x in ctr]
    k = [int(x) & _MASK for x in key]
    for rnd in range(10):
        p0 = _M0 * c[0]
        p1 = _M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & _MASK, p1 & _MASK,
             ((p0 >> 32) ^ c[3] ^ k[1]) & _MASK, p0 & _MASK]
        if rnd < 9:
            k = [(k[0] + _W0) & _MASK, (k[1] + _W1) & _MASK]
    return c


def element_random_word(P, worker, step, seed):
    quad = P >> 2
    out = philox4x32_10([quad & _MASK, quad >> 32, worker, step], [seed & _MASK, seed >> 32])
    return out[P & 3]


def scaled_magnitude(g, N, b):
    """a = min(fl32(|g| * fl32(s/N)), s) as an exact Fraction plus floor and fractional part."""
    s = np.float32((1 << b) - 1)
    scale = np.float32(s / np.float32(N))
    a = min(np.float32(abs(np.float32(g))) * scale, s)
    fa = Fraction(float(np.float32(a)))
    lo = fa.numerator // fa.denominator
    return fa, lo, fa - lo


def round_up_probability(p):
    """P[u < p] for u uniform on {0, 1, ..., 2^24 - 1} / 2^24: ceil(p * 2^24) / 2^24."""
    scaled = p * (1 << 24)
    ceil = -((-scaled.numerator) // scaled.denominator)
    return Fraction(ceil, 1 << 24)


def quantize_element(g, N, b, P, worker, step, seed):
    """(sign, level) of one element straight from Eq. (5)-(6) with the repository's conventions."""
    sign = 1 if np.signbit(np.float32(g)) else 0
    if not (np.float32(N) >= np.float32(2.0 ** -100)):
        return sign, 0
    _, lo, p = scaled_magnitude(g, N, b)
    u = Fraction(element_random_word(P, worker, step, seed) >> 8, 1 << 24)
    return sign, lo + (1 if u < p else 0)


def single_width_rule_agrees(got, want, n_seg, factor, b_min, b_max):
    """Validity check for a (b, G-bar) pair against the oracle's when the two sides may add a worker's
    sum_l N_l^2 (Lemma 1's G-bar_t^2) in different orders.  Each binary64 sum of n_seg non-negative
    terms is within (n_seg - 1) * 2^-53 relative of the exact one, so G-bar (a square root: half the
    relative error, plus the roundings of the mean and the root) agrees to (n_seg + 4) * 2^-53
    relative.  The widths must be equal unless s* = factor * G-bar lies within that relative distance
    of a level count 2^b - 1 (Eq. (17) rounded up), where either neighbouring width is correct."""
    (b_got, g_got), (b_want, g_want) = got, want
    rel = (n_seg + 4) * 2.0 ** -53
    if abs(g_got - g_want) > rel * g_want:
        return False
    if b_got == b_want:
        return True
    lo, hi = sorted((int(b_got), int(b_want)))
    levels = float((1 << lo) - 1)
    return hi == lo + 1 and b_min <= lo and hi <= b_max and abs(factor * g_want - levels) <= 2 * rel * levels


def rule_factor(t, T, eps_hat_q, alpha):
    """sqrt(T/eps_hat_q) * alpha^((T-1-t)/2), the factor of Eq. (17) in front of G-bar."""
    return (T / eps_hat_q) ** 0.5 * alpha ** ((T - 1 - t) / 2.0)
