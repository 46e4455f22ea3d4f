"""Pins for the sign-only baseline (Table 2's SignSGD row: one bit per element, no norm)."""
import numpy as np

from tests.test_oracle_loop_pieces import _table2, ITERS, W


def _layout(oracle, seg):
    dp = oracle.padded_elems(seg)
    valid = np.zeros(dp, dtype=bool)
    for st, n in zip(oracle.seg_starts(seg), seg):
        valid[st:st + n] = True
    return dp, valid


def test_sign_plane_is_numpy_signbit_packed_little_endian(oracle):
    rng = np.random.default_rng(60)
    seg = [130, 0, 1, 1000, 64]
    dp, valid = _layout(oracle, seg)
    g = rng.standard_normal((3, dp)).astype(np.float32)
    g[0, 5] = -0.0
    g[1, 6] = 0.0
    g[:, ~valid] = -1.0                                         # pads never set a bit
    msg = oracle.sign_pack(seg, g)
    want = np.packbits(np.signbit(g) & valid, axis=1, bitorder="little")
    assert msg.shape == (3, dp // 8) and np.array_equal(msg, want)
    assert (msg[0, 0] >> 5) & 1 == 1 and (msg[1, 0] >> 6) & 1 == 0   # -0.0 is negative, +0.0 is not


def test_sign_plane_equals_the_quantizers_sign_plane(oracle):
    rng = np.random.default_rng(61)
    seg = [300, 77]
    dp, _ = _layout(oracle, seg)
    g = (rng.standard_normal((2, dp)) * 1e-2).astype(np.float32)
    full = oracle.quantize_pack(seg, g, oracle.norm(seg, g), 3, 1, 0)
    assert np.array_equal(oracle.sign_pack(seg, g), full[:, :dp // 8])


def test_mean_and_majority_against_numpy(oracle):
    rng = np.random.default_rng(62)
    seg = [200, 5, 129]
    dp, valid = _layout(oracle, seg)
    for M in (1, 2, 5, 8):
        g = rng.standard_normal((M, dp)).astype(np.float32)
        msg = oracle.sign_pack(seg, g)
        sgn = np.where(np.signbit(g), -1.0, 1.0) * valid
        assert np.array_equal(oracle.sign_reduce(seg, msg), (sgn.sum(axis=0) / M).astype(np.float32))
        assert np.array_equal(oracle.sign_reduce(seg, msg, majority=True), np.sign(sgn.sum(axis=0)).astype(np.float32))
        scales = rng.uniform(0.1, 2.0, size=(M, 3)).astype(np.float32)
        per_elem = np.zeros((M, dp))
        for l, (st, n) in enumerate(zip(oracle.seg_starts(seg), seg)):
            per_elem[:, st:st + n] = scales[:, l:l + 1].astype(np.float64)
        want = ((sgn * per_elem).sum(axis=0) / M).astype(np.float32)
        got = oracle.sign_reduce(seg, msg, scales=scales)
        assert np.allclose(got, want, rtol=1e-7, atol=0)
    # even M: a tie gives 0
    g = np.ones((2, 128), dtype=np.float32)
    g[1] = -1
    assert np.all(oracle.sign_reduce([128], oracle.sign_pack([128], g), majority=True) == 0)


def test_scaled_sign_with_mean_abs_scale_keeps_the_l1_norm(oracle):
    """With c = mean|g| (the scaled-sign compressor) one worker's decoded vector has the l1 norm of g."""
    rng = np.random.default_rng(63)
    g = rng.standard_normal((1, 1024)).astype(np.float32)
    c = np.abs(g).mean(dtype=np.float64)
    out = oracle.sign_reduce([1024], oracle.sign_pack([1024], g), scales=np.array([[c]], dtype=np.float32))
    assert abs(np.abs(out).sum(dtype=np.float64) - np.abs(g).sum(dtype=np.float64)) < 1e-3
    assert np.array_equal(np.signbit(out), np.signbit(g[0]))


def test_message_size_is_table2s_signsgd_cost(oracle):
    """D'/8 bytes per worker = d bits when d is a multiple of 128; times W*T it is the SignSGD row."""
    rows = _table2()
    sgd, sign = rows["VanillaSGD"][1], rows["SignSGD"][1]
    for col, (task, T) in enumerate(ITERS.items()):
        d = round(sgd[col] * 2 ** 30 * 8 / (W * T * 32))
        d128 = d // 128 * 128
        assert oracle.sign_pack([d128], np.zeros((1, d128), dtype=np.float32)).shape[1] * 8 == d128
        gib = W * T * d / 8 / 2 ** 30
        assert abs(gib - sign[col]) < 0.006
        assert oracle.comm_cost_bits(W, d, 0, 0, 32) * T / 8 / 2 ** 30 == gib
