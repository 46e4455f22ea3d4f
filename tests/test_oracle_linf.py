"""Pins for the p = infinity choice of the norm in Eq. (5) and the bit rule (Eq. (17)) that goes
with it.  The quantizer itself is unchanged (it takes the norms as an input), so the pins here
cover the norm, the rule's G-bar, and what the max norm buys: ratios |g_j|/N that never exceed 1
and, with one level bit, the ternary scheme of the related work."""
import numpy as np

from tests import pyref

SEED = 0xD05C6D


def test_norm_linf_against_numpy(oracle):
    rng = np.random.default_rng(31)
    seg = [1000, 3, 129, 70000, 0, 1]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    M = 4
    grads = (rng.standard_t(3, size=(M, dp)) * 3e-3).astype(np.float32)
    norms = oracle.norm_linf(seg, grads)
    for i in range(M):
        for l, (st, n) in enumerate(zip(starts, seg)):
            want = np.abs(grads[i, st:st + n]).max() if n else np.float32(0)
            assert norms[i, l] == want                    # a max is exact: no rounding to allow for
    poisoned = grads.copy()
    valid = np.zeros(dp, dtype=bool)
    for st, n in zip(starts, seg):
        valid[st:st + n] = True
    poisoned[:, ~valid] = np.inf                          # pads are not part of the tensor
    assert np.array_equal(oracle.norm_linf(seg, poisoned), norms)


def test_norm_linf_hand_vectors(oracle):
    g = np.zeros((1, 128), dtype=np.float32)
    g[0, :4] = [0.5, -3.0, 2.0, -0.0]
    assert oracle.norm_linf([4], g)[0, 0] == 3.0          # the largest magnitude, sign dropped
    assert oracle.norm_linf([1], g)[0, 0] == 0.5
    assert oracle.norm_linf([3, 1], np.concatenate([g, g], axis=1)).tolist() == [[3.0, 0.5]]
    g[0, :4] = [1e-40, -2e-40, 0, 0]                      # subnormals compare like any number
    assert oracle.norm_linf([4], g)[0, 0] == np.float32(2e-40)
    g[0, :4] = [1.0, np.nan, -2.0, 0.5]                   # a NaN element is skipped
    assert oracle.norm_linf([4], g)[0, 0] == 2.0
    g[0, :4] = 0
    assert oracle.norm_linf([4], g)[0, 0] == 0.0


def test_linf_is_below_l2_and_above_rms(oracle):
    """||g||_inf <= ||g||_2 <= sqrt(d) ||g||_inf for every vector."""
    rng = np.random.default_rng(32)
    seg = [777, 64, 5000]
    dp = oracle.padded_elems(seg)
    grads = rng.standard_normal((3, dp)).astype(np.float32)
    n2 = oracle.norm(seg, grads).astype(np.float64)
    ninf = oracle.norm_linf(seg, grads).astype(np.float64)
    d = np.array(seg, dtype=np.float64)
    assert np.all(ninf <= n2 * (1 + 1e-7))
    assert np.all(n2 <= np.sqrt(d) * ninf * (1 + 1e-7))


def test_select_bits_linf_uses_the_largest_segment_norm(oracle):
    """G-bar^2 = (1/M) sum_i (max_l N_il)^2, then Eq. (17) as printed, rounded up."""
    rng = np.random.default_rng(33)
    T, alpha = 40, 0.9
    for _ in range(300):
        M, n_seg = int(rng.integers(1, 9)), int(rng.integers(1, 6))
        norms = rng.uniform(0.01, 2.0, size=(M, n_seg)).astype(np.float32)
        t = int(rng.integers(0, T))
        eps = float(10 ** rng.uniform(-4, 1))
        gbar_want = np.sqrt((norms.astype(np.float64).max(axis=1) ** 2).mean())
        b, gbar = oracle.select_bits_linf(norms, t, T, eps, alpha, 1, 8)
        assert abs(gbar - gbar_want) <= 1e-12 * gbar_want
        s_star = np.sqrt(T / eps) * alpha ** ((T - 1 - t) / 2.0) * gbar_want
        b_paper = np.log2(s_star + 1) + 1
        if abs(b_paper - round(b_paper)) < 1e-9:
            continue
        assert b == int(np.clip(np.ceil(b_paper) - 1, 1, 8))


def test_select_bits_linf_special_cases(oracle):
    """One segment: the two rules coincide.  n_seg equal segment norms: the p = 2 rule sees a norm
    sqrt(n_seg) larger, the p = infinity rule does not."""
    norms = np.array([[0.3], [0.5], [0.1]], dtype=np.float32)
    for t in (0, 10, 19):
        assert oracle.select_bits_linf(norms, t, 20, 0.3, 0.9, 1, 8) == oracle.select_bits(norms, t, 20, 0.3, 0.9, 1, 8)
    same = np.full((4, 9), 0.25, dtype=np.float32)
    _, g2 = oracle.select_bits(same, 5, 20, 0.3, 0.9, 1, 8)
    _, ginf = oracle.select_bits_linf(same, 5, 20, 0.3, 0.9, 1, 8)
    assert abs(ginf - 0.25) < 1e-12 and abs(g2 - 0.75) < 1e-12


def test_linf_bound_of_lemma1_with_segment_scales(oracle):
    """With one scale per segment the variance of the quantized gradient is at most
    sum_l d_l N_l^2/(4 s^2) <= d max_l N_l^2/(4 s^2): the G-bar the rule uses is large enough for
    Lemma 1.  Monte-Carlo over steps on a two-segment vector."""
    rng = np.random.default_rng(34)
    seg = [256, 384]
    dp = oracle.padded_elems(seg)
    g = np.zeros((1, dp), dtype=np.float32)
    g[0, :256] = rng.standard_normal(256) * 0.1
    g[0, 256:] = rng.standard_normal(384) * 0.02
    norms = oracle.norm_linf(seg, g)
    b, draws = 2, 1500
    s = (1 << b) - 1
    err2 = 0.0
    for step in range(draws):
        sign, level = oracle.quantize(seg, g, norms, b, SEED, step)
        q = oracle.dequant_reduce(seg, sign, level, norms, b)
        err2 += float(((q.astype(np.float64) - g[0]) ** 2).sum())
    var = err2 / draws
    per_segment = (256 * float(norms[0, 0]) ** 2 + 384 * float(norms[0, 1]) ** 2) / (4 * s * s)
    whole = 640 * float(norms.max()) ** 2 / (4 * s * s)
    assert var <= per_segment <= whole
    assert var > 0.2 * per_segment          # and the bound is not vacuous for this input


def test_max_element_gets_the_top_level_and_no_ratio_exceeds_one(oracle):
    """N = max|g| a power of two: s/N and |g|*(s/N) are exact, so the largest element sits on
    level s with probability 1 and every other element below it."""
    rng = np.random.default_rng(35)
    d = 640
    g = rng.uniform(-1, 1, size=(1, d)).astype(np.float32) * np.float32(0.24)
    g[0, 17] = -0.25
    norms = oracle.norm_linf([d], g)
    assert norms[0, 0] == 0.25
    for b in (1, 3, 8):
        s = (1 << b) - 1
        for step in range(20):
            sign, level = oracle.quantize([d], g, norms, b, SEED, step)
            assert level[0, 17] == s and sign[0, 17] == 1
            assert level.max() == s
            exact = np.abs(g[0].astype(np.float64)) * s / 0.25
            assert np.all(level[0] >= np.floor(exact)) and np.all(level[0] <= np.floor(exact) + 1)


def test_one_level_bit_with_max_norm_is_the_ternary_scheme(oracle):
    """b = 1 and N = max|g|: each element becomes sgn(g_j) * N with probability |g_j|/N, else 0.
    Checked element by element against the rule written out with the Python Philox twin."""
    g = np.zeros((1, 128), dtype=np.float32)
    vals = np.array([0.5, -1.0, 0.25, 0.0, -0.75, 0.125, 1.0, -0.3], dtype=np.float32)
    g[0, :8] = vals
    norms = oracle.norm_linf([8], g)
    assert norms[0, 0] == 1.0
    for step in range(64):
        sign, level = oracle.quantize([8], g, norms, 1, SEED, step, worker_base=3)
        q = oracle.dequant_reduce([8], sign, level, norms, 1)
        for P, v in enumerate(vals):
            u = (pyref.element_random_word(P, 3, step, SEED) >> 8) / 2.0 ** 24
            keep = u < abs(float(v))                     # N = 1, s = 1: p_r = |g_j|
            want = np.sign(v) * 1.0 if keep and abs(v) < 1 else (np.sign(v) if abs(v) == 1 else 0.0)
            assert q[P] == np.float32(want)
