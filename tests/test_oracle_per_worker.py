"""Pins for per-worker (and per-worker-per-tensor) bit-widths: the rule with the worker's own norm
in Eq. (17), messages of different lengths in one step, the average with a unit per worker and
tensor."""
import numpy as np

SEED = 0xD05C6D


def _kappa(T, eps, alpha, t):
    return np.sqrt(T / eps) * alpha ** ((T - 1 - t) / 2.0)


def test_real_valued_rule_meets_the_constraint_with_equality():
    """with s*_{t,i} = kappa_t N_{t,i} the constraint sum_t alpha^(T-1-t) (1/M) sum_i N_{t,i}^2/s_{t,i}^2
    equals eps_hat whatever the workers' norms (the single-width term Gbar^2/s^2 is its equal-s case)"""
    T, eps, alpha, M = 20, 0.3, 0.92, 5
    rng = np.random.default_rng(0)
    total = 0.0
    for t in range(T):
        N = rng.uniform(0.01, 3.0, size=M)
        s = _kappa(T, eps, alpha, t) * N
        total += alpha ** (T - 1 - t) * float((N ** 2 / s ** 2).mean())
    assert abs(total - eps) < 1e-12
    # equal s for all workers: the same expression is Gbar^2 / s^2
    N = rng.uniform(0.01, 3.0, size=M)
    assert abs((N ** 2 / 4.0 ** 2).mean() - (N ** 2).mean() / 16.0) < 1e-15


def test_proportional_levels_minimise_the_cost_between_two_workers():
    """brute force: min log2 s_1 + log2 s_2 on (N_1^2/s_1^2 + N_2^2/s_2^2)/2 = c is at s_i = N_i/sqrt(c)"""
    for N1, N2 in [(0.3, 1.7), (2.0, 0.05)]:
        c, best = 0.01, None
        for theta in np.linspace(1e-4, 1 - 1e-4, 200001):
            s1 = np.sqrt(N1 ** 2 / (2 * theta * c))
            s2 = np.sqrt(N2 ** 2 / (2 * (1 - theta) * c))
            cost = np.log2(s1) + np.log2(s2)
            if best is None or cost < best[0]:
                best = (cost, s1, s2)
        assert abs(best[1] - N1 / np.sqrt(c)) < 2e-3 * N1 / np.sqrt(c)
        assert abs(best[2] - N2 / np.sqrt(c)) < 2e-3 * N2 / np.sqrt(c)


def test_rule_is_eq17_with_the_workers_own_norm(oracle):
    rng = np.random.default_rng(1)
    T, alpha = 40, 0.9
    for _ in range(200):
        M, n_seg = int(rng.integers(1, 9)), int(rng.integers(1, 6))
        norms = rng.uniform(0.01, 2.0, size=(M, n_seg)).astype(np.float32)
        t = int(rng.integers(0, T))
        eps = float(10 ** rng.uniform(-4, 1))
        b = oracle.select_bits_per_worker(norms, t, T, eps, alpha, 1, 8)
        bt = oracle.select_bits_per_worker(norms, t, T, eps, alpha, 1, 8, per_tensor=True)
        for i in range(M):
            # one worker alone is the single-width rule (Gbar = its norm); its tensors alone, the per-tensor rule
            want, _ = oracle.select_bits(norms[i:i + 1], t, T, eps, alpha, 1, 8)
            assert np.all(b[i] == want)
            want_t, _ = oracle.select_bits_per_tensor(norms[i:i + 1], t, T, eps, alpha, 1, 8)
            assert np.array_equal(bt[i], want_t)
            assert np.all(bt[i] <= b[i])
        N = np.sqrt((norms.astype(np.float64) ** 2).sum(axis=1))
        b_paper = np.log2(_kappa(T, eps, alpha, t) * N + 1) + 1
        for i in range(M):
            if abs(b_paper[i] - round(b_paper[i])) > 1e-9:
                assert b[i, 0] == int(np.clip(np.ceil(b_paper[i]) - 1, 1, 8))


def test_workers_with_equal_norms_get_the_shared_width(oracle):
    norms = np.tile(np.array([[0.3, 0.7, 0.05]], dtype=np.float32), (6, 1))
    for t in (0, 9, 19):
        b_all, _ = oracle.select_bits(norms, t, 20, 0.02, 0.9, 1, 8)
        assert np.all(oracle.select_bits_per_worker(norms, t, 20, 0.02, 0.9, 1, 8) == b_all)
        bt, _ = oracle.select_bits_per_tensor(norms, t, 20, 0.02, 0.9, 1, 8)
        assert np.all(oracle.select_bits_per_worker(norms, t, 20, 0.02, 0.9, 1, 8, per_tensor=True) == bt)


def test_ceiling_keeps_the_error_budget(oracle):
    T, eps, alpha, M = 30, 0.05, 0.95, 4
    rng = np.random.default_rng(2)
    total = 0.0
    for t in range(T):
        norms = rng.uniform(0.05, 0.4, size=(M, 1)).astype(np.float32)
        b = oracle.select_bits_per_worker(norms, t, T, eps, alpha, 1, 8)
        assert np.all(b < 8)
        s = (1 << b[:, 0].astype(np.int64)) - 1
        total += alpha ** (T - 1 - t) * float((norms[:, 0].astype(np.float64) ** 2 / s ** 2).mean())
    assert total <= eps


def test_messages_are_each_workers_own_per_tensor_message(oracle):
    rng = np.random.default_rng(3)
    seg = [200, 0, 129, 3000]
    dp = oracle.padded_elems(seg)
    M = 4
    grads = (rng.standard_normal((M, dp)) * 1e-2).astype(np.float32)
    norms = oracle.norm(seg, grads)
    b = rng.integers(1, 9, size=(M, 4)).astype(np.int32)
    packed = oracle.quantize_pack_w(seg, grads, norms, b, SEED, 6, worker_base=2)
    assert packed.shape[1] == max(oracle.packed_bytes_v(seg, b[i]) for i in range(M))
    for i in range(M):
        alone = oracle.quantize_pack_v(seg, grads[i:i + 1], norms[i:i + 1], b[i], SEED, 6, worker_base=2 + i)
        n = alone.shape[1]
        assert np.array_equal(packed[i, :n], alone[0]) and np.all(packed[i, n:] == 0)
    # equal rows: the shared per-tensor message
    same = np.tile(b[:1], (M, 1))
    assert np.array_equal(oracle.quantize_pack_w(seg, grads, norms, same, SEED, 6),
                          oracle.quantize_pack_v(seg, grads, norms, b[0], SEED, 6))


def test_average_uses_a_unit_per_worker_and_tensor(oracle):
    """two workers, one 128-element tensor, widths 1 and 3, norms chosen so both units are exact"""
    rng = np.random.default_rng(4)
    seg = [128]
    grads = np.zeros((2, 128), dtype=np.float32)
    grads[0] = rng.choice([-2.0, 0.0, 2.0], size=128)             # N/s = 2/1 with N = 2 passed in
    grads[1] = rng.integers(-7, 8, size=128).astype(np.float32)   # N/s = 7/7
    norms = np.array([[2.0], [7.0]], dtype=np.float32)
    b = np.array([[1], [3]], dtype=np.int32)
    packed = oracle.quantize_pack_w(seg, grads, norms, b, SEED, 0)
    out = oracle.unpack_dequant_reduce_w(seg, packed, norms, b)
    assert np.array_equal(out, ((grads[0] + grads[1]) / 2).astype(np.float32))   # grid values: no rounding noise
    # with the roles of the widths swapped the decode is wrong: the unit really is per worker
    wrong = oracle.unpack_dequant_reduce_w(seg, packed, norms, b[::-1].copy())
    assert not np.array_equal(wrong, out)


def test_unbiased_with_unequal_widths(oracle):
    rng = np.random.default_rng(5)
    seg = [300, 212]
    dp = oracle.padded_elems(seg)
    M = 3
    grads = (rng.standard_normal((M, dp)) * 0.05).astype(np.float32)
    grads[:, 300:384] = 0
    norms = oracle.norm(seg, grads)
    b = np.array([[1, 4], [3, 2], [8, 1]], dtype=np.int32)
    draws, mean = 1200, np.zeros(dp)
    var_bound = 0.0
    for i in range(M):
        for l, n in enumerate(seg):
            var_bound += n * float(norms[i, l]) ** 2 / (4.0 * ((1 << b[i, l]) - 1) ** 2) / M ** 2
    err2 = 0.0
    true_mean = grads.astype(np.float64).mean(axis=0)
    for step in range(draws):
        q = oracle.unpack_dequant_reduce_w(seg, oracle.quantize_pack_w(seg, grads, norms, b, SEED, step), norms, b)
        mean += q
        err2 += float(((q - true_mean) ** 2).sum())
    assert err2 / draws <= var_bound                                   # (1/M^2) sum_i sum_l d_l N_il^2/(4 s_il^2)
    assert np.abs(mean / draws - true_mean).max() < 5 * np.sqrt(var_bound / draws)
