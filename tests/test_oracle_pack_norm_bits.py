"""Pins for the oracle's message layout, norm, bit rule (Eq. (17)) and server average."""
from fractions import Fraction

import numpy as np
import pytest

SEED = 0xD05C6D


# ---------------------------------------------------------------- message layout (wire format)
@pytest.mark.parametrize("b", range(1, 9))
def test_pack_matches_little_endian_bit_arrays(oracle, b):
    """Sign plane = bit P of a little-endian bit array; level plane = element P at bits
    [P*b, P*b+b), LSB first.  Rebuilt here with numpy.packbits, a library routine."""
    rng = np.random.default_rng(b)
    dp = 128 * 5
    sign = rng.integers(0, 2, size=dp, dtype=np.uint8)
    level = rng.integers(0, 1 << b, size=dp, dtype=np.uint8)
    packed = oracle.pack(sign, level, b)
    assert packed.size == dp // 8 + dp * b // 8
    want_sign = np.packbits(sign, bitorder="little")
    bits = ((level[:, None] >> np.arange(b, dtype=np.uint8)) & 1).astype(np.uint8).reshape(-1)
    want_level = np.packbits(bits, bitorder="little")
    assert np.array_equal(packed[:dp // 8], want_sign)
    assert np.array_equal(packed[dp // 8:], want_level)
    s2, l2 = oracle.unpack(packed, dp, b)
    assert np.array_equal(s2, sign) and np.array_equal(l2, level)


def test_pack_special_widths(oracle):
    """b = 8 is one byte per element, b = 4 two nibbles per byte (low nibble first), and the sign
    plane read as 64-bit little-endian words has element 64w+k at bit k."""
    dp = 256
    level = np.arange(dp, dtype=np.uint8)
    sign = (np.arange(dp) % 3 == 0).astype(np.uint8)
    p8 = oracle.pack(sign, level, 8)
    assert np.array_equal(p8[dp // 8:], level)
    lv4 = level & 15
    p4 = oracle.pack(sign, lv4, 4)
    assert np.array_equal(p4[dp // 8:], lv4[0::2] | (lv4[1::2] << 4))
    words = p4[:dp // 8].view("<u8")
    for w in range(dp // 64):
        for k in range(64):
            assert (int(words[w]) >> k) & 1 == sign[64 * w + k]


def test_message_size_is_the_cost_of_eq7(oracle):
    """Eq. (7): d*b_paper bits per worker per step with b_paper = b + 1 (plus B_pre for the norm,
    which travels beside the message).  With d a multiple of 128 there is no padding."""
    d = 128 * 77
    for b in range(1, 9):
        assert 8 * oracle.packed_bytes([d], b) == d * (b + 1)
    assert oracle.padded_elems([1, 128, 129, 0]) == 128 + 128 + 256 + 0
    assert list(oracle.seg_starts([1, 128, 129, 5])) == [0, 128, 256, 512]


# ---------------------------------------------------------------------------------------- norm
def test_norm_against_numpy(oracle):
    rng = np.random.default_rng(3)
    seg = [1000, 3, 129, 70000]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    M = 4
    grads = (rng.standard_normal((M, dp)) * np.float32(3e-3)).astype(np.float32)
    norms = oracle.norm(seg, grads)
    for i in range(M):
        for l, (st, n) in enumerate(zip(starts, seg)):
            want = np.linalg.norm(grads[i, st:st + n].astype(np.float64))
            assert abs(float(norms[i, l]) - want) <= np.spacing(np.float32(want))
    # pads are ignored: poison them
    poisoned = grads.copy()
    valid = np.zeros(dp, dtype=bool)
    for st, n in zip(starts, seg):
        valid[st:st + n] = True
    poisoned[:, ~valid] = np.nan
    assert np.array_equal(oracle.norm(seg, poisoned), norms)


def test_norm_exact_vectors(oracle):
    g = np.zeros((1, 128), dtype=np.float32)
    g[0, :2] = [3.0, 4.0]
    assert oracle.norm([2], g)[0, 0] == 5.0
    g[0, :4] = [2.0, -2.0, 2.0, -2.0]
    assert oracle.norm([4], g)[0, 0] == 4.0
    g[0, :3] = [1e-20, 0, 0]     # squares underflow in binary32 but not in binary64
    assert oracle.norm([1], g)[0, 0] == np.float32(1e-20)


# ------------------------------------------------------------------------------ bit rule Eq. 17
def _s_star(T, eps, alpha, t, gbar):
    return np.sqrt(T / eps) * alpha ** ((T - 1 - t) / 2.0) * gbar


def test_real_valued_rule_meets_the_constraint_with_equality():
    """With the real-valued s*_t of Eq. (17), each step contributes eps_hat/T to the constraint of
    Eq. (16): sum_t alpha^(T-1-t) G_t^2 / s*_t^2 = eps_hat.  (Pure mathematics of the paper; fixes
    the formula the oracle must implement, including the exponent (T-1-t)/2.)"""
    T, eps, alpha = 50, 0.37, 0.93
    rng = np.random.default_rng(0)
    gbar = rng.uniform(0.1, 3.0, size=T)
    total = sum(alpha ** (T - 1 - t) * gbar[t] ** 2 / _s_star(T, eps, alpha, t, gbar[t]) ** 2 for t in range(T))
    assert abs(total - eps) < 1e-12


def test_select_bits_is_ceiling_of_eq17(oracle):
    """b = smallest integer with 2^b - 1 >= s*  <=>  b_paper = ceil(log2(s*+1) + 1) with b = b_paper - 1."""
    rng = np.random.default_rng(1)
    T, alpha = 40, 0.9
    for _ in range(300):
        M, n_seg = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        norms = rng.uniform(0.01, 2.0, size=(M, n_seg)).astype(np.float32)
        t = int(rng.integers(0, T))
        eps = float(10 ** rng.uniform(-4, 1))
        gbar_want = np.sqrt((norms.astype(np.float64) ** 2).sum() / M)
        b, gbar = oracle.select_bits(norms, t, T, eps, alpha, 1, 8)
        assert abs(gbar - gbar_want) <= 1e-12 * gbar_want
        s_star = _s_star(T, eps, alpha, t, gbar_want)
        b_paper = np.log2(s_star + 1) + 1                    # Eq. (17) as printed
        if abs(b_paper - round(b_paper)) < 1e-9:
            continue                                         # on an integer boundary: either side
        want = int(np.clip(np.ceil(b_paper) - 1, 1, 8))
        assert b == want


def test_ceiling_keeps_the_error_budget(oracle):
    """Rounding up keeps sum_t alpha^(T-1-t) G_t^2/(2^b_t - 1)^2 <= eps_hat when no step is clamped."""
    T, eps, alpha = 30, 0.05, 0.95
    rng = np.random.default_rng(2)
    total = 0.0
    for t in range(T):
        norms = rng.uniform(0.05, 0.4, size=(4, 2)).astype(np.float32)
        b, gbar = oracle.select_bits(norms, t, T, eps, alpha, 1, 8)
        assert 1 <= b < 8
        total += alpha ** (T - 1 - t) * gbar ** 2 / ((1 << b) - 1) ** 2
    assert total <= eps


def test_select_bits_monotone_and_clamped(oracle):
    T, alpha, eps = 100, 0.97, 1e-2
    base = np.full((4, 3), 0.02, dtype=np.float32)
    # more bits as training proceeds (t up), as gradients grow, as the budget tightens
    bs_t = [oracle.select_bits(base, t, T, eps, alpha, 1, 8)[0] for t in range(T)]
    assert all(x <= y for x, y in zip(bs_t, bs_t[1:])) and bs_t[0] < bs_t[-1]
    bs_g = [oracle.select_bits(base * k, 50, T, eps, alpha, 1, 8)[0] for k in (0.1, 0.5, 1, 2, 8, 64)]
    assert all(x <= y for x, y in zip(bs_g, bs_g[1:])) and bs_g[0] < bs_g[-1]
    bs_e = [oracle.select_bits(base, 50, T, e, alpha, 1, 8)[0] for e in (10, 1, 1e-1, 1e-2, 1e-4, 1e-6)]
    assert all(x <= y for x, y in zip(bs_e, bs_e[1:])) and bs_e[0] < bs_e[-1]
    assert oracle.select_bits(base * 1e6, 50, T, eps, alpha, 2, 8)[0] == 8
    assert oracle.select_bits(base * 1e-9, 50, T, eps, alpha, 2, 8)[0] == 2
    # alpha = 1 and constant gradients: constant b
    assert len({oracle.select_bits(base, t, T, eps, 1.0, 1, 8)[0] for t in range(0, T, 7)}) == 1


def test_ratio_test_of_the_discussion(oracle):
    """G_{t+1}/G_t = sqrt(alpha) leaves s* unchanged; a faster decay lowers b, a slower one raises
    it (Section 5, 'Dynamic Adjustment in the Number of Bits')."""
    T, alpha, eps = 64, 0.95, 1.58e-3
    g0 = 0.5
    seq_eq = [g0 * np.sqrt(alpha) ** t for t in range(T)]
    b_eq = {oracle.select_bits(np.array([[g]], dtype=np.float32), t, T, eps, alpha, 1, 8)[0] for t, g in enumerate(seq_eq)}
    assert len(b_eq) == 1
    fast = [oracle.select_bits(np.array([[g0 * 0.8 ** t]], dtype=np.float32), t, T, eps, alpha, 1, 8)[0] for t in range(20)]
    slow = [oracle.select_bits(np.array([[g0 * 0.99 ** t]], dtype=np.float32), t, T, eps, alpha, 1, 8)[0] for t in range(40)]
    assert fast[0] > fast[-1] and all(x >= y for x, y in zip(fast, fast[1:]))
    assert slow[0] < slow[-1] and all(x <= y for x, y in zip(slow, slow[1:]))


def test_select_bits_rejects_bad_arguments(oracle):
    n = np.ones((2, 2), dtype=np.float32)
    for kw in (dict(t=-1), dict(t=10), dict(T=0), dict(eps_hat_q=0.0), dict(alpha=0.0), dict(alpha=1.5),
               dict(b_min=0), dict(b_max=9), dict(b_min=5, b_max=4)):
        args = dict(t=0, T=10, eps_hat_q=1.0, alpha=0.9, b_min=1, b_max=8)
        args.update(kw)
        with pytest.raises(ValueError):
            oracle.select_bits(n, **args)


# ------------------------------------------------------------------------------ server average
def test_average_exact_with_power_of_two_units(oracle):
    """All N_i = s*2^e: units are 2^e and the average is an exact integer computation."""
    rng = np.random.default_rng(4)
    b, e, M, d = 4, -12, 8, 500
    s = 15
    dp = oracle.padded_elems([d])
    sign = np.zeros((M, dp), dtype=np.uint8)
    level = np.zeros((M, dp), dtype=np.uint8)
    sign[:, :d] = rng.integers(0, 2, size=(M, d))
    level[:, :d] = rng.integers(0, s + 1, size=(M, d))
    norms = np.full((M, 1), s * 2.0 ** e, dtype=np.float32)
    out = oracle.dequant_reduce([d], sign, level, norms, b)
    signed = level.astype(np.int64) * (1 - 2 * sign.astype(np.int64))
    want = np.array([float(Fraction(int(x), M) * Fraction(2) ** e) for x in signed.sum(axis=0)])
    assert np.array_equal(out.astype(np.float64), want)


def test_average_of_one_worker_is_plain_dequantization(oracle):
    rng = np.random.default_rng(6)
    seg = [300, 77]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    grads = (rng.standard_normal((1, dp)) * 1e-2).astype(np.float32)
    norms = oracle.norm(seg, grads)
    b = 5
    sign, level = oracle.quantize(seg, grads, norms, b, SEED, 0)
    out = oracle.dequant_reduce(seg, sign, level, norms, b)
    for l, (st, n) in enumerate(zip(starts, seg)):
        unit = norms[0, l] / np.float32(31)
        want = level[0, st:st + n].astype(np.float32) * unit * np.where(sign[0, st:st + n] == 1, np.float32(-1), np.float32(1))
        assert np.array_equal(out[st:st + n], want)


def test_average_converges_to_the_mean_gradient(oracle):
    """Eq. (10): the aggregate of many workers' quantized copies of the same g approaches g."""
    rng = np.random.default_rng(8)
    d, M, b = 256, 512, 3
    g = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    grads = np.tile(g, (M, 1))
    norms = oracle.norm([d], grads)
    packed = oracle.quantize_pack([d], grads, norms, b, SEED, 3)
    out = oracle.unpack_dequant_reduce([d], packed, norms, b)
    unit = float(norms[0, 0]) / 7
    assert np.max(np.abs(out - g)) <= 5 * 0.5 * unit / np.sqrt(M)


def test_messages_round_trip_through_both_passes(oracle):
    rng = np.random.default_rng(10)
    seg = [1, 127, 128, 129, 4096 + 5]
    dp = oracle.padded_elems(seg)
    M = 5
    grads = (rng.laplace(size=(M, dp)) * 1e-3).astype(np.float32)
    norms = oracle.norm(seg, grads)
    for b in range(1, 9):
        sign, level = oracle.quantize(seg, grads, norms, b, SEED, b)
        nbytes = oracle.packed_bytes(seg, b)
        packed = oracle.quantize_pack(seg, grads, norms, b, SEED, b, packed_stride=nbytes + 48)
        for i in range(M):
            s2, l2 = oracle.unpack(packed[i], dp, b)
            assert np.array_equal(s2, sign[i]) and np.array_equal(l2, level[i])
            assert not packed[i, nbytes:].any()
        a = oracle.dequant_reduce(seg, sign, level, norms, b)
        c = oracle.unpack_dequant_reduce(seg, packed, norms, b)
        assert np.array_equal(a, c)


def test_range_forms_equal_slices_of_the_whole(oracle):
    rng = np.random.default_rng(12)
    seg = [300, 0, 5, 1000, 129]
    dp = oracle.padded_elems(seg)
    M, b = 3, 5
    grads = (rng.standard_normal((M, dp)) * 1e-2).astype(np.float32)
    norms = oracle.norm(seg, grads)
    sign, level = oracle.quantize(seg, grads, norms, b, SEED, 4, worker_base=2)
    out = oracle.dequant_reduce(seg, sign, level, norms, b)
    for p0, p1 in ((0, 128), (256, 1024), (dp - 256, dp), (0, dp), (384, 384)):
        sl = np.ascontiguousarray(grads[:, p0:p1]) if p1 > p0 else np.zeros((M, 1), dtype=np.float32)[:, :0].copy()
        if p1 == p0:
            continue
        s2, l2 = oracle.quantize_range(seg, sl, norms, b, SEED, 4, p0, p1, worker_base=2)
        assert np.array_equal(s2, sign[:, p0:p1]) and np.array_equal(l2, level[:, p0:p1])
        o2 = oracle.dequant_reduce_range(seg, s2, l2, norms, b, p0, p1)
        assert np.array_equal(o2, out[p0:p1])


def test_gbar_is_the_plain_index_order_sum_of_lemma_1(oracle):
    """G-bar_t^2 = (1/M) sum_i ||g^(i)||^2 with ||g^(i)||^2 = sum_l N_{i,l}^2 (Lemma 1): the oracle adds a
    worker's squares one after the other in index order in binary64 -- no blocks, no pairing.  Checked on
    5000 tensors against exact rational arithmetic (the running sum's error bound) and against the same
    running sum spelled out in Python floats; on some of the inputs a sum taken in blocks of 1024 gives a
    different G-bar, so the check can tell the two orders apart."""
    from fractions import Fraction
    n_seg, M = 5000, 2
    told_apart = 0
    for seed in range(12):
        rng = np.random.default_rng(770 + seed)
        norms = (10 ** rng.uniform(-6, 2, size=(M, n_seg))).astype(np.float32)
        _, gbar = oracle.select_bits(norms, 0, 10, 1.0, 0.9, 1, 8)
        if seed == 0:
            exact = sum(Fraction(float(x)) ** 2 for x in norms.reshape(-1)) / M
            assert abs(Fraction(gbar) ** 2 - exact) <= exact * n_seg * Fraction(1, 2 ** 52)
        total = blocked = 0.0
        for i in range(M):
            worker = 0.0
            for x in norms[i]:
                worker += float(x) * float(x)
            total += worker
            worker = 0.0
            for base in range(0, n_seg, 1024):
                blk = 0.0
                for x in norms[i, base:base + 1024]:
                    blk += float(x) * float(x)
                worker += blk
            blocked += worker
        assert gbar == float(np.sqrt(total / M)), seed
        told_apart += float(np.sqrt(blocked / M)) != gbar
    assert told_apart >= 1
