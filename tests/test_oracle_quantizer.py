"""Pins for the oracle's EWU quantizer (Eq. (5)-(6)) that do not use the oracle to check itself:
exact outcome probabilities on tiny vectors, Monte-Carlo unbiasedness (Eq. (10)) and the Lemma 1
variance bound, grid reproduction, the zero vector, deterministic invariants, special cases."""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

from tests import pyref

SEED = 0xD05C6D


def _norm32(g):
    return np.float32(np.sqrt(np.sum(g.astype(np.float64) ** 2)))


def _draws(oracle, g, b, n_workers, n_steps, N=None):
    """levels[n_steps*n_workers][d], signs: the same vector quantized under many (worker, step)."""
    d = g.size
    dp = oracle.padded_elems([d])
    grads = np.zeros((n_workers, dp), dtype=np.float32)
    grads[:, :d] = g
    N = _norm32(g) if N is None else np.float32(N)
    norms = np.full((n_workers, 1), N, dtype=np.float32)
    levels = []
    for step in range(n_steps):
        sign, level = oracle.quantize([d], grads, norms, b, SEED, step)
        levels.append(level[:, :d].copy())
    return np.concatenate(levels, axis=0), sign[:, :d], N


@pytest.mark.parametrize("b", [1, 2, 4, 7])
@pytest.mark.parametrize("g", [
    np.array([0.3, -0.7, 0.2, 0.61], dtype=np.float32),
    np.array([1e-3, -2e-3, 5e-4], dtype=np.float32),
    np.array([0.6, 0.8], dtype=np.float32),
    np.array([-0.123], dtype=np.float32),
])
def test_outcome_frequencies_match_exact_enumeration(oracle, g, b):
    """All 2^d floor/ceil outcomes with probabilities prod p_j^x_j (1-p_j)^(1-x_j) (Eq. (6)),
    computed in exact rational arithmetic, against the oracle's empirical joint frequencies; and
    the exact distribution itself is unbiased and meets the per-element variance of Lemma 1."""
    d = g.size
    N = _norm32(g)
    s = (1 << b) - 1
    lo, p = [], []
    for x in g:
        a, l, frac = pyref.scaled_magnitude(x, N, b)
        lo.append(l)
        p.append(pyref.round_up_probability(frac))
        # E[zeta] = a/s exactly up to the 2^-24 lattice of u (Appendix A, first display)
        assert abs((l + p[-1]) - a) < Fraction(1, 1 << 24)
    n_workers, n_steps = 2048, 32
    levels, sign, _ = _draws(oracle, g, b, n_workers, n_steps)
    n = levels.shape[0]
    assert np.array_equal(sign[0], np.signbit(g).astype(np.uint8))
    for outcome in product([0, 1], repeat=d):
        prob = Fraction(1)
        for j, x in enumerate(outcome):
            prob *= p[j] if x else 1 - p[j]
        want = np.array([lo[j] + outcome[j] for j in range(d)], dtype=np.uint8)
        got = int(np.all(levels == want, axis=1).sum())
        pf = float(prob)
        sigma = np.sqrt(max(pf * (1 - pf), 1e-12) * n)
        assert abs(got - pf * n) <= 5 * sigma + 1, (outcome, got, pf * n)
    # exact variance per element: p(1-p)/s^2 <= 1/(4 s^2)  (Appendix A, second display)
    for pj in p:
        assert pj * (1 - pj) / (s * s) <= Fraction(1, 4 * s * s)


@pytest.mark.parametrize("b", [1, 3, 4, 8])
def test_monte_carlo_unbiased_and_lemma1_variance(oracle, b):
    """E[Q(g)] = g (Eq. (10)) and E||Q(g)||^2 - ||g||^2 <= d ||g||^2 / (4 s^2) (Lemma 1)."""
    rng = np.random.default_rng(100 + b)
    d = 64
    g = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    s = (1 << b) - 1
    levels, sign, N = _draws(oracle, g, b, 4096, 32)
    n = levels.shape[0]
    unit = float(N) / s
    sgn = np.where(np.signbit(g), -1.0, 1.0)
    q = levels.astype(np.float64) * unit * sgn
    mean = q.mean(axis=0)
    sd = q.std(axis=0)
    assert np.all(np.abs(mean - g) <= 5 * sd / np.sqrt(n) + 1e-7 * float(N))
    excess = (q ** 2).sum(axis=1).mean() - float((g.astype(np.float64) ** 2).sum())
    bound = d * float(N) ** 2 / (4 * s * s)
    assert excess <= bound * 1.02
    # the exact trace of the variance: (N/s)^2 sum p_j (1-p_j)
    pj = np.array([float(pyref.scaled_magnitude(x, N, b)[2]) for x in g])
    want = unit ** 2 * np.sum(pj * (1 - pj))
    assert abs(excess - want) <= 0.05 * want + 1e-12


@pytest.mark.parametrize("b", range(1, 9))
def test_grid_values_are_reproduced_exactly(oracle, b):
    """N = s*2^e and g_j = +-l_j*2^e make scale = 2^-e and a = l_j exactly, so p_r = 0: the level is
    l_j under every seed and dequantization returns g bit for bit."""
    s = (1 << b) - 1
    e = -9
    rng = np.random.default_rng(b)
    d = 300
    lev = rng.integers(0, s + 1, size=d)
    sgn = rng.choice([-1.0, 1.0], size=d)
    g = (lev * sgn * 2.0 ** e).astype(np.float32)
    N = np.float32(s * 2.0 ** e)
    dp = oracle.padded_elems([d])
    grads = np.zeros((3, dp), dtype=np.float32)
    grads[:, :d] = g
    norms = np.full((3, 1), N, dtype=np.float32)
    for step in (0, 1, 99):
        sign, level = oracle.quantize([d], grads, norms, b, SEED + step, step)
        assert np.array_equal(level[:, :d], np.broadcast_to(lev.astype(np.uint8), (3, d)))
        assert np.array_equal(sign[:, :d], np.broadcast_to(np.signbit(g).astype(np.uint8), (3, d)))
        out = oracle.dequant_reduce([d], sign, level, norms, b)
        assert np.array_equal(out[:d].view(np.uint32) & 0x7FFFFFFF, g.view(np.uint32) & 0x7FFFFFFF)
        assert np.array_equal(out[:d][lev > 0], g[lev > 0])
        assert np.all(out[d:] == 0)


def test_zero_vector(oracle):
    d = 200
    dp = oracle.padded_elems([d])
    grads = np.zeros((2, dp), dtype=np.float32)
    norms = oracle.norm([d], grads)
    assert np.all(norms == 0)
    sign, level = oracle.quantize([d], grads, norms, 4, SEED, 0)
    assert not sign.any() and not level.any()
    packed = oracle.quantize_pack([d], grads, norms, 4, SEED, 0)
    assert not packed.any()
    out = oracle.unpack_dequant_reduce([d], packed, norms, 4)
    assert np.array_equal(out.view(np.uint32), np.zeros(dp, dtype=np.uint32))  # exactly +0.0


@pytest.mark.parametrize("bad", [0.0, 1e-35, np.nan, -1.0])
def test_unusable_norm_takes_the_zero_path(oracle, bad):
    d = 130
    rng = np.random.default_rng(5)
    dp = oracle.padded_elems([d])
    grads = np.zeros((1, dp), dtype=np.float32)
    grads[0, :d] = rng.standard_normal(d)
    norms = np.array([[bad]], dtype=np.float32)
    sign, level = oracle.quantize([d], grads, norms, 3, SEED, 1)
    assert not level.any()
    assert np.array_equal(sign[0, :d], np.signbit(grads[0, :d]).astype(np.uint8))
    out = oracle.dequant_reduce([d], sign, level, norms, 3)
    assert np.all(out == 0)


@pytest.mark.parametrize("b", range(1, 9))
def test_deterministic_invariants(oracle, b):
    """level in {floor(a), floor(a)+1}, level <= s, |Q(g)_j - g_j| <= N/s, pads encode as zero."""
    rng = np.random.default_rng(40 + b)
    seg = [257, 1, 128, 1000]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    M = 3
    grads = (rng.standard_t(3, size=(M, dp)) * 1e-3).astype(np.float32)  # pads hold garbage
    norms = oracle.norm(seg, grads)
    s = (1 << b) - 1
    sign, level = oracle.quantize(seg, grads, norms, b, SEED, 2)
    valid = np.zeros(dp, dtype=bool)
    for l, (st, n) in enumerate(zip(starts, seg)):
        valid[st:st + n] = True
        for i in range(M):
            x = grads[i, st:st + n]
            N = norms[i, l]
            a = np.minimum(np.abs(x) * (np.float32(s) / N), np.float32(s))
            fl = np.floor(a).astype(np.int64)
            lv = level[i, st:st + n].astype(np.int64)
            assert np.all((lv == fl) | (lv == fl + 1))
            assert lv.max() <= s
            q = lv * (float(N) / s) * np.where(np.signbit(x), -1.0, 1.0)
            assert np.all(np.abs(q - x) <= float(N) / s * (1 + 2.0 ** -22))
    assert not sign[:, ~valid].any() and not level[:, ~valid].any()


def test_one_hot_vector_clamps_to_s(oracle):
    """|g_j|/||g|| can round above 1; the level must still be <= s."""
    for val in (0.1, 3.0000002, 1e-30, 7.3e20):
        g = np.array([val], dtype=np.float32)
        N = _norm32(g)
        for b in (1, 4, 8):
            levels, _, _ = _draws(oracle, g, b, 8, 2, N=np.nextafter(N, np.float32(0)))
            assert np.all(levels == (1 << b) - 1)


def test_b1_is_ternary_stochastic_sign(oracle):
    """s = 1: level in {0,1} with P[1] = |g_j|/N -- the textbook ternary quantizer."""
    g = np.array([0.5, -0.25, 0.75, 0.1], dtype=np.float32)
    N = np.float32(1.0)
    levels, _, _ = _draws(oracle, g, 1, 4096, 16, N=N)
    assert set(np.unique(levels)) <= {0, 1}
    freq = levels.mean(axis=0)
    n = levels.shape[0]
    want = np.abs(g)
    assert np.all(np.abs(freq - want) <= 5 * np.sqrt(want * (1 - want) / n))


def test_python_twin_agrees_element_by_element(oracle):
    """Second implementation (Python floats/Fractions, big-integer Philox) gives the same codes,
    including the counter layout {P>>2, worker, step} and the word choice P&3."""
    rng = np.random.default_rng(9)
    seg = [37, 130]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    M = 3
    grads = (rng.standard_normal((M, dp)) * 1e-2).astype(np.float32)
    norms = oracle.norm(seg, grads)
    for b in (2, 5):
        sign, level = oracle.quantize(seg, grads, norms, b, SEED, 7, worker_base=10)
        for i in range(M):
            for l, (st, n) in enumerate(zip(starts, seg)):
                for P in range(st, st + n):
                    sg, lv = pyref.quantize_element(grads[i, P], norms[i, l], b, int(P), 10 + i, 7, SEED)
                    assert (sign[i, P], level[i, P]) == (sg, lv)


def test_steps_workers_and_seeds_decorrelate(oracle):
    g = np.full(512, 0.5 / np.sqrt(512), dtype=np.float32)  # a = 0.5*s/sqrt(d)... p well inside (0,1)
    dp = oracle.padded_elems([512])
    grads = np.tile(g, (2, 1))
    norms = np.full((2, 1), 1.0, dtype=np.float32)
    _, l0 = oracle.quantize([512], grads, norms, 6, 1, 0)
    _, l1 = oracle.quantize([512], grads, norms, 6, 1, 1)
    _, l2 = oracle.quantize([512], grads, norms, 6, 2, 0)
    assert (l0[0] != l0[1]).mean() > 0.2      # workers differ
    assert (l0[0] != l1[0]).mean() > 0.2      # steps differ
    assert (l0[0] != l2[0]).mean() > 0.2      # seeds differ
    _, l0b = oracle.quantize([512], grads, norms, 6, 1, 0)
    assert np.array_equal(l0, l0b)            # and the draw is reproducible
    _, lw = oracle.quantize([512], grads[1:], norms[1:], 6, 1, 0, worker_base=1)
    assert np.array_equal(lw[0], l0[1])       # worker ids are global


def test_round_up_threshold_is_strict_and_24_bit(oracle):
    """With N = s the scale is exactly 1 and a = p = g for g in [0,1).  Place g exactly on the
    element's own uniform u = (r>>8)/2^24 (r from the big-integer Philox): u < p is false there,
    and true one lattice step above -- so the comparison is strict and u has 24 bits."""
    b = 3
    N = np.float32(7.0)
    step, worker = 5, 2
    d = 48
    dp = oracle.padded_elems([d])
    u = np.array([pyref.element_random_word(P, worker, step, SEED) >> 8 for P in range(d)], dtype=np.int64)
    assert (u & 1).any() and not (u & 1).all()
    for delta, want in ((0, 0), (1, 1), (-1, 0)):
        g = np.zeros((1, dp), dtype=np.float32)
        g[0, :d] = ((u + delta).astype(np.float64) * 2.0 ** -24).astype(np.float32)
        ok = (u + delta > 0) & (u + delta < (1 << 24))
        _, level = oracle.quantize([d], g, np.array([[N]], dtype=np.float32), b, SEED, step, worker_base=worker)
        assert np.all(level[0, :d][ok] == want)


def test_norm_smaller_than_an_element_still_clamps(oracle):
    """The norm is an input: if it is too small for the data (a = 2s here) the level stays s."""
    g = np.zeros((1, 128), dtype=np.float32)
    g[0, :3] = [0.5, -1.0, 0.25]
    for b in (1, 4, 8):
        s = (1 << b) - 1
        _, level = oracle.quantize([3], g, np.array([[0.5]], dtype=np.float32), b, SEED, 0)
        assert level[0, 0] == s and level[0, 1] == s
        assert level[0, 2] in (s // 2, s // 2 + 1)


@pytest.mark.parametrize("center", [1 << 32, 1 << 34, (1 << 36) + (1 << 34)])
def test_python_twin_agrees_beyond_32_bit_indices(oracle, center):
    """Padded indices past 2^32 (the index no longer fits a 32-bit word) and past 2^34 (the quad
    index P>>2 reaches the counter's second word): the oracle's codes for a window around the
    boundary equal the Python twin's, element by element."""
    rng = np.random.default_rng(center % 1000003)
    seg = [center + 4096]
    p0, p1 = center - 128, center + 128
    M = 2
    g = (rng.standard_normal((M, p1 - p0)) * 0.05).astype(np.float32)
    norms = np.array([[1.0], [0.75]], dtype=np.float32)
    for b in (1, 4, 8):
        sign, level = oracle.quantize_range(seg, g, norms, b, SEED, 3, p0, p1, worker_base=4)
        for i in range(M):
            for j in range(p1 - p0):
                sg, lv = pyref.quantize_element(g[i, j], norms[i, 0], b, p0 + j, 4 + i, 3, SEED)
                assert (sign[i, j], level[i, j]) == (sg, lv), (b, i, p0 + j)
    # the two sides of the 2^34 boundary really draw from different counters
    if center == 1 << 34:
        lo = pyref.element_random_word(center - 4, 0, 0, SEED)
        assert pyref.philox4x32_10([(center - 4) >> 2 & 0xFFFFFFFF, 0, 0, 0], [SEED & 0xFFFFFFFF, SEED >> 32])[0] == lo
        assert pyref.element_random_word(center, 0, 0, SEED) == \
            pyref.philox4x32_10([0, 1, 0, 0], [SEED & 0xFFFFFFFF, SEED >> 32])[0]


@pytest.mark.parametrize("b", [1, 3, 4, 8])
def test_level_never_grows_with_the_norm(oracle, b):
    """For a fixed element, seed, step and worker the level of Eq. (5)-(6) is a non-increasing
    function of the norm (all roundings included): scale, scaled magnitude, clamp and the stochastic
    step are each monotone.  Hence a level that is the same for two norms is the level for every
    norm between them -- what the one-pass path with bracketed norms relies on.  Checked on sweeps of
    the norm that include neighbouring binary32 values and norms near the largest element."""
    rng = np.random.default_rng(700 + b)
    d = 4096
    g = np.concatenate([rng.standard_normal(d // 2) * 1e-2, rng.standard_t(3, d // 2) * 1e-2]).astype(np.float32)
    g[:8] = [0.0, -0.0, 1e-30, -1e-30, 5.0, -5.0, np.float32(1e-2), np.float32(-1e-2)]
    grads = g[None, :]
    base = float(np.sqrt((g.astype(np.float64) ** 2).sum()))
    sweep = [np.float32(base * f) for f in (0.01, 0.1, 0.5, 0.875, 0.99, 1.0, 1.01, 1.125, 2.0, 10.0, 1000.0)]
    for f in (0.5, 1.0, 5.0):                       # runs of neighbouring floats
        x = np.float32(base * f)
        for _ in range(12):
            sweep.append(x)
            x = np.nextafter(x, np.float32(np.inf))
    sweep += [np.float32(5.0), np.nextafter(np.float32(5.0), np.float32(0)), np.float32(4.0)]   # |g|/N at and above 1
    sweep = sorted(set(float(x) for x in sweep))
    prev = None
    for N in sweep:
        _, level = oracle.quantize([d], grads, np.array([[N]], dtype=np.float32), b, SEED, 5, worker_base=3)
        if prev is not None:
            assert np.all(level[0] <= prev), N
        prev = level[0].copy()
    # every binary32 norm of three runs of 2048 consecutive values, on a short vector
    short = np.ascontiguousarray(grads[:, :128])
    for f in (0.31, 1.0, 2.7):
        x = np.float32(base * f)
        prev = None
        for _ in range(2048):
            _, level = oracle.quantize([128], short, np.array([[x]], dtype=np.float32), b, SEED, 5, worker_base=3)
            if prev is not None:
                assert np.all(level[0] <= prev), float(x)
            prev = level[0].copy()
            x = np.nextafter(x, np.float32(np.inf))
    # equal at both ends => equal inside
    lo, hi = np.float32(base * 0.875), np.float32(base * 1.125)
    _, l_lo = oracle.quantize([d], grads, np.array([[lo]], dtype=np.float32), b, SEED, 5, worker_base=3)
    _, l_hi = oracle.quantize([d], grads, np.array([[hi]], dtype=np.float32), b, SEED, 5, worker_base=3)
    same = l_lo[0] == l_hi[0]
    for f in rng.uniform(0.875, 1.125, size=20):
        N = np.float32(base * f)
        if not (lo <= N <= hi):
            continue
        _, l_mid = oracle.quantize([d], grads, np.array([[N]], dtype=np.float32), b, SEED, 5, worker_base=3)
        assert np.array_equal(l_mid[0][same], l_lo[0][same])
        assert np.all((l_mid[0] <= l_lo[0]) & (l_mid[0] >= l_hi[0]))
