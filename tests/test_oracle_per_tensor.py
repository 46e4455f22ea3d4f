"""Pins for the per-tensor bit-widths: the rule (the Lagrangian argument of the paper's appendix
"Proof of Eq. (17)" carried out with one level count per tensor), the message layout with widths
that change from tensor to tensor, the codes and the average."""
import numpy as np
import pytest

SEED = 0xD05C6D


# --------------------------------------------------------------------------------------- the rule
def _kappa(T, eps, alpha, t):
    return np.sqrt(T / eps) * alpha ** ((T - 1 - t) / 2.0)


def test_real_valued_rule_meets_the_constraint_with_equality():
    """s*_{t,l} = sqrt(T/eps) alpha^((T-1-t)/2) Nbar_{t,l} makes
    sum_t alpha^(T-1-t) sum_l (d_l/d) Nbar_{t,l}^2 / s*_{t,l}^2 = eps for any tensor sizes."""
    T, eps, alpha = 25, 0.21, 0.9
    rng = np.random.default_rng(0)
    d = np.array([100.0, 7.0, 3000.0, 64.0])
    total = 0.0
    for t in range(T):
        nbar = rng.uniform(0.01, 2.0, size=4)
        s = _kappa(T, eps, alpha, t) * nbar
        total += alpha ** (T - 1 - t) * float(((d / d.sum()) * nbar ** 2 / s ** 2).sum())
    assert abs(total - eps) < 1e-12


def test_proportional_levels_minimise_the_cost_under_the_appendix_approximation():
    """With 2^(b-1) ~ s (the approximation of the appendix) the cost of one iteration is
    sum_l d_l log2 s_l + const.  Brute force over two tensors: among all (s_1, s_2) on the
    constraint (d_1/d) N_1^2/s_1^2 + (d_2/d) N_2^2/s_2^2 = c the cheapest has s_1/s_2 = N_1/N_2,
    whatever the sizes."""
    for d1, d2, N1, N2 in [(100.0, 900.0, 0.3, 1.7), (5000.0, 10.0, 2.0, 0.05), (1.0, 1.0, 1.0, 3.0)]:
        d, c = d1 + d2, 0.01
        best = None
        # parametrise the constraint by the share theta of the budget spent on tensor 1
        for theta in np.linspace(1e-4, 1 - 1e-4, 200001):
            s1 = np.sqrt((d1 / d) * N1 ** 2 / (theta * c))
            s2 = np.sqrt((d2 / d) * N2 ** 2 / ((1 - theta) * c))
            cost = d1 * np.log2(s1) + d2 * np.log2(s2)
            if best is None or cost < best[0]:
                best = (cost, s1, s2)
        assert abs(best[1] / best[2] - N1 / N2) < 2e-3 * N1 / N2
        # and its scale is the rule's: s_l = Nbar_l / sqrt(c)
        assert abs(best[1] - N1 / np.sqrt(c)) < 2e-3 * N1 / np.sqrt(c)


def test_rule_is_eq17_with_the_tensor_norm(oracle):
    rng = np.random.default_rng(1)
    T, alpha = 40, 0.9
    for _ in range(200):
        M, n_seg = int(rng.integers(1, 9)), int(rng.integers(1, 7))
        norms = rng.uniform(0.01, 2.0, size=(M, n_seg)).astype(np.float32)
        t = int(rng.integers(0, T))
        eps = float(10 ** rng.uniform(-4, 1))
        b, nbar = oracle.select_bits_per_tensor(norms, t, T, eps, alpha, 1, 8)
        want_nbar = np.sqrt((norms.astype(np.float64) ** 2).mean(axis=0))
        assert np.allclose(nbar, want_nbar, rtol=1e-12, atol=0)
        for l in range(n_seg):
            b_paper = np.log2(_kappa(T, eps, alpha, t) * want_nbar[l] + 1) + 1      # Eq. (17) as printed
            if abs(b_paper - round(b_paper)) < 1e-9:
                continue
            assert b[l] == int(np.clip(np.ceil(b_paper) - 1, 1, 8))
            # a tensor alone is the single-width rule
            assert b[l] == oracle.select_bits(norms[:, l:l + 1], t, T, eps, alpha, 1, 8)[0]


def test_no_tensor_gets_more_bits_than_the_single_width(oracle):
    """Nbar_l <= Gbar, so b_l <= b for every tensor; zero tensors sit at b_min."""
    rng = np.random.default_rng(2)
    for _ in range(200):
        M, n_seg = 4, int(rng.integers(2, 12))
        norms = (10 ** rng.uniform(-4, 0.5, size=(M, n_seg))).astype(np.float32)
        norms[:, 0] = 0
        t, T = int(rng.integers(0, 30)), 30
        b_all, _ = oracle.select_bits(norms, t, T, 1e-3, 0.95, 2, 8)
        b, _ = oracle.select_bits_per_tensor(norms, t, T, 1e-3, 0.95, 2, 8)
        assert np.all(b <= b_all) and b[0] == 2


def test_ceiling_keeps_the_error_budget(oracle):
    T, eps, alpha = 30, 0.05, 0.95
    rng = np.random.default_rng(3)
    d = np.array([400.0, 30.0, 2000.0])
    total = 0.0
    for t in range(T):
        norms = rng.uniform(0.05, 0.4, size=(4, 3)).astype(np.float32)
        b, nbar = oracle.select_bits_per_tensor(norms, t, T, eps, alpha, 1, 8)
        assert np.all(b < 8)
        s = (1 << b.astype(np.int64)) - 1
        total += alpha ** (T - 1 - t) * float(((d / d.sum()) * nbar ** 2 / s ** 2).sum())
    assert total <= eps


def test_rule_rejects_bad_arguments(oracle):
    n = np.ones((2, 3), dtype=np.float32)
    for bad in [dict(t=5, T=5), dict(eps_hat_q=0.0), dict(alpha=1.5), dict(b_min=0), dict(b_max=9), dict(b_min=5, b_max=4)]:
        args = dict(t=0, T=5, eps_hat_q=0.1, alpha=0.9, b_min=1, b_max=8)
        args.update(bad)
        with pytest.raises(Exception):
            oracle.select_bits_per_tensor(n, **args)


# ----------------------------------------------------------------------------------- the message
def _random_codes(rng, seg, widths):
    dp = sum(-(-n // 128) * 128 for n in seg)
    sign = rng.integers(0, 2, size=dp, dtype=np.uint8)
    level = np.zeros(dp, dtype=np.uint8)
    st = 0
    for n, b in zip(seg, widths):
        pad = -(-n // 128) * 128
        level[st:st + pad] = rng.integers(0, 1 << b, size=pad, dtype=np.uint8)
        st += pad
    return dp, sign, level


def test_pack_v_is_the_tensors_bit_arrays_one_after_another(oracle):
    rng = np.random.default_rng(4)
    seg, widths = [130, 1, 0, 700, 128], [3, 8, 5, 1, 6]
    dp, sign, level = _random_codes(rng, seg, widths)
    msg = oracle.pack_v(sign, level, seg, widths)
    assert msg.size == oracle.packed_bytes_v(seg, widths) == dp // 8 + (256 * 3 + 128 * 8 + 0 + 768 * 1 + 128 * 6) // 8
    assert np.array_equal(msg[:dp // 8], np.packbits(sign, bitorder="little"))
    bits = []
    st = 0
    for n, b in zip(seg, widths):
        pad = -(-n // 128) * 128
        fields = (level[st:st + pad, None] >> np.arange(b)) & 1          # least significant bit first
        bits.append(fields.reshape(-1).astype(np.uint8))
        st += pad
    assert np.array_equal(msg[dp // 8:], np.packbits(np.concatenate(bits), bitorder="little"))
    sg, lv = oracle.unpack_v(msg, seg, widths)
    assert np.array_equal(sg, sign) and np.array_equal(lv, level)


def test_equal_widths_give_the_uniform_message(oracle):
    rng = np.random.default_rng(5)
    seg = [300, 5, 1000]
    for b in (1, 4, 7):
        dp, sign, level = _random_codes(rng, seg, [b] * 3)
        assert np.array_equal(oracle.pack_v(sign, level, seg, [b] * 3), oracle.pack(sign, level, b))
        assert oracle.packed_bytes_v(seg, [b] * 3) == oracle.packed_bytes(seg, b)


def test_every_tensor_region_starts_on_a_16_byte_boundary(oracle):
    rng = np.random.default_rng(6)
    for _ in range(50):
        n_seg = int(rng.integers(1, 10))
        seg = [int(x) for x in rng.integers(0, 1000, size=n_seg)]
        widths = [int(x) for x in rng.integers(1, 9, size=n_seg)]
        off = 0
        for n, b in zip(seg, widths):
            assert off % 16 == 0
            off += -(-n // 128) * 128 * b // 8
        assert oracle.packed_bytes_v(seg, widths) == oracle.padded_elems(seg) // 8 + off


def test_cost_per_tensor_matches_eq7(oracle):
    seg, widths = [1000, 24, 512], [2, 8, 4]
    assert oracle.comm_cost_bits_per_tensor(8, seg, widths, 32) == 8 * (1000 * 3 + 24 * 9 + 512 * 5 + 3 * 32)
    for b in (1, 5):
        assert oracle.comm_cost_bits_per_tensor(4, seg, [b] * 3, 32) == oracle.comm_cost_bits(4, sum(seg), b, 3, 32)
    # the message carries the same bits, padding aside
    seg128 = [1024, 128, 512]
    assert oracle.packed_bytes_v(seg128, widths) * 8 == oracle.comm_cost_bits_per_tensor(1, seg128, widths, 0)


# ------------------------------------------------------------------------- codes and the average
def test_codes_are_the_uniform_codes_tensor_by_tensor(oracle):
    rng = np.random.default_rng(7)
    seg, widths = [200, 0, 129, 3000, 64], [2, 4, 8, 1, 5]
    dp = oracle.padded_elems(seg)
    starts = oracle.seg_starts(seg)
    M = 3
    grads = (rng.standard_normal((M, dp)) * 1e-2).astype(np.float32)
    norms = oracle.norm(seg, grads)
    sign, level = oracle.quantize_v(seg, grads, norms, widths, SEED, 11, worker_base=4)
    for st, n, b in zip(starts, seg, widths):
        sg_u, lv_u = oracle.quantize(seg, grads, norms, b, SEED, 11, worker_base=4)
        pad = -(-n // 128) * 128
        assert np.array_equal(sign[:, st:st + pad], sg_u[:, st:st + pad])
        assert np.array_equal(level[:, st:st + pad], lv_u[:, st:st + pad])
        assert level[:, st:st + pad].max(initial=0) <= (1 << b) - 1
    # range form = slice of the whole
    sg_r, lv_r = oracle.quantize_v_range(seg, np.ascontiguousarray(grads[:, 256:3584]), norms, widths, SEED, 11,
                                         256, 3584, worker_base=4)
    assert np.array_equal(sg_r, sign[:, 256:3584]) and np.array_equal(lv_r, level[:, 256:3584])


def test_average_uses_each_tensors_own_unit(oracle):
    """norms powers of two and s_l from the tensor's width: one worker, out = +-level * N_l / s_l."""
    seg, widths = [128, 128, 128], [1, 2, 4]
    dp = 384
    rng = np.random.default_rng(8)
    _, sign, level = _random_codes(rng, seg, widths)
    norms = np.array([[3.0, 1.5, 30.0]], dtype=np.float32)           # / s = 3, 0.5, 2 exactly
    out = oracle.dequant_reduce_v(seg, sign[None], level[None], norms, widths)
    unit = np.repeat(np.array([3.0, 0.5, 2.0]), 128)
    want = np.where(sign == 1, -1.0, 1.0) * level * unit
    assert np.array_equal(out, want.astype(np.float32))
    uniform = oracle.dequant_reduce(seg, sign[None], level[None], norms, 2)
    assert np.array_equal(out[128:256], uniform[128:256])
    part = oracle.dequant_reduce_v_range(seg, sign[None, 128:], level[None, 128:], norms, widths, 128, 384)
    assert np.array_equal(part, out[128:])


def test_variance_bound_with_per_tensor_levels(oracle):
    """E||Q(g) - g||^2 <= sum_l d_l N_l^2 / (4 s_l^2), the form of Lemma 1 the rule is built on."""
    rng = np.random.default_rng(9)
    seg, widths = [256, 640], [3, 1]
    dp = oracle.padded_elems(seg)
    g = np.zeros((1, dp), dtype=np.float32)
    g[0, :256] = rng.standard_normal(256) * 0.02
    g[0, 256:] = rng.standard_normal(640) * 0.3
    norms = oracle.norm(seg, g)
    draws, err2, mean = 1500, 0.0, np.zeros(dp)
    for step in range(draws):
        msg = oracle.quantize_pack_v(seg, g, norms, widths, SEED, step)
        q = oracle.unpack_dequant_reduce_v(seg, msg, norms, widths).astype(np.float64)
        err2 += float(((q - g[0]) ** 2).sum())
        mean += q
    bound = sum(n * float(N) ** 2 / (4.0 * ((1 << b) - 1) ** 2) for n, N, b in zip(seg, norms[0], widths))
    assert err2 / draws <= bound
    assert np.abs(mean / draws - g[0]).max() < 5 * np.sqrt(bound / draws)    # unbiased


def test_messages_round_trip_through_both_passes(oracle):
    rng = np.random.default_rng(10)
    seg, widths = [77, 1000, 0, 130], [8, 3, 2, 6]
    dp = oracle.padded_elems(seg)
    M = 4
    grads = (rng.standard_normal((M, dp)) * 1e-3).astype(np.float32)
    norms = oracle.norm(seg, grads)
    msg = oracle.quantize_pack_v(seg, grads, norms, widths, SEED, 2)
    sign, level = oracle.quantize_v(seg, grads, norms, widths, SEED, 2)
    for i in range(M):
        assert np.array_equal(msg[i], oracle.pack_v(sign[i], level[i], seg, widths))
    assert np.array_equal(oracle.unpack_dequant_reduce_v(seg, msg, norms, widths),
                          oracle.dequant_reduce_v(seg, sign, level, norms, widths))
