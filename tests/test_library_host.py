"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, its host logic
(layout queries, the bit rule, argument validation) agrees with the oracle.  No kernel runs."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dq():
    import paper_2107_14575_amd as dq
    if not os.path.exists(dq.library_path()):
        from paper_2107_14575_amd import build
        build.build_library()
    dq.load_library()
    return dq


def test_library_exports_every_declared_symbol(dq):
    header = open(os.path.join(ROOT, "include", "dq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dq_[a-z_0-9]+)\s*\(", header))
    assert {"dq_norm", "dq_select_bits", "dq_quantize_pack", "dq_unpack_dequant_reduce"} <= declared
    lib = dq.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    from paper_2107_14575_amd import binding
    assert declared == set(binding.EXPORTS)


def test_layout_queries_match_the_oracle(dq, oracle):
    rng = np.random.default_rng(0)
    for _ in range(50):
        n_seg = int(rng.integers(1, 12))
        seg = [int(x) for x in rng.choice([0, 1, 5, 127, 128, 129, 1000, 4096, 70001], size=n_seg)]
        plan = dq.Plan(seg)
        assert plan.n_seg == n_seg
        assert plan.padded_elems == oracle.padded_elems(seg)
        assert [plan.segment_start(l) for l in range(n_seg)] == list(oracle.seg_starts(seg))
        for b in range(1, 9):
            assert plan.packed_bytes(b) == oracle.packed_bytes(seg, b)
        assert plan.packed_bytes(0) == -1 and plan.packed_bytes(9) == -1
        assert plan.workspace_bytes(4) >= 16 and plan.workspace_bytes(0) == -1
        assert plan.segment_start(n_seg) == -1
        plan.close()


def test_select_bits_bit_exact_against_the_oracle(dq, oracle):
    rng = np.random.default_rng(1)
    for _ in range(3000):
        M, n_seg = int(rng.integers(1, 17)), int(rng.integers(1, 8))
        norms = (10 ** rng.uniform(-6, 1, size=(M, n_seg))).astype(np.float32)
        T = int(rng.integers(1, 1000))
        t = int(rng.integers(0, T))
        eps = float(10 ** rng.uniform(-8, 2))
        alpha = float(rng.uniform(0.5, 1.0))
        b_min = int(rng.integers(1, 9))
        b_max = int(rng.integers(b_min, 9))
        got = dq.select_bits(norms, t, T, eps, alpha, b_min, b_max)
        want = oracle.select_bits(norms, t, T, eps, alpha, b_min, b_max)
        assert got[0] == want[0]
        assert abs(got[1] - want[1]) <= 1e-15 * want[1]
        got = dq.select_bits_linf(norms, t, T, eps, alpha, b_min, b_max)
        want = oracle.select_bits_linf(norms, t, T, eps, alpha, b_min, b_max)
        assert got[0] == want[0]
        assert abs(got[1] - want[1]) <= 1e-15 * want[1]


def test_select_bits_rejects_bad_arguments(dq):
    n = np.ones((2, 2), dtype=np.float32)
    good = dict(t=0, T=10, eps_hat_q=1.0, alpha=0.9, b_min=1, b_max=8)
    assert dq.select_bits(n, **good)[0] >= 1
    for kw in (dict(t=-1), dict(t=10), dict(T=0), dict(eps_hat_q=0.0), dict(eps_hat_q=float("nan")),
               dict(alpha=0.0), dict(alpha=1.5), dict(b_min=0), dict(b_max=9), dict(b_min=5, b_max=4)):
        args = dict(good)
        args.update(kw)
        with pytest.raises(dq.DQError) as e:
            dq.select_bits(n, **args)
        assert e.value.status == -1


def test_plan_create_rejects_bad_arguments(dq):
    lib = dq.load_library()
    h = C.c_void_p()
    lens = (C.c_int64 * 2)(5, -1)
    assert lib.dq_plan_create(lens, 2, C.byref(h)) == -1 and not h.value
    assert lib.dq_plan_create(lens, 0, C.byref(h)) == -1
    assert lib.dq_plan_create(None, 1, C.byref(h)) == -1
    lib.dq_plan_destroy(None)  # harmless
    assert lib.dq_status_string(0) == b"ok" and b"invalid" in lib.dq_status_string(-1)


def test_device_entry_points_validate_before_touching_a_gpu(dq):
    """Null pointers and bad sizes are rejected with DQ_ERR_INVALID_ARG whether or not a GPU is
    present (nothing is launched)."""
    lib = dq.load_library()
    plan = dq.Plan([1000])
    h = plan.handle
    fake = 0x1000  # aligned, never dereferenced on these paths
    assert lib.dq_norm(h, None, 1024, 1, fake, fake, None) == -1
    assert lib.dq_norm(h, fake, 1000, 1, fake, fake, None) == -1            # stride < D'
    assert lib.dq_norm(h, fake, 1024, 0, fake, fake, None) == -1            # M < 1
    assert lib.dq_norm(h, fake + 4, 1024, 1, fake, fake, None) == -1        # misaligned
    assert lib.dq_quantize_pack(h, fake, 1024, 1, fake, 0, 1, 0, 0, fake, 4096, None) == -1   # b = 0
    assert lib.dq_quantize_pack(h, fake, 1024, 1, fake, 9, 1, 0, 0, fake, 4096, None) == -1   # b = 9
    assert lib.dq_quantize_pack(h, fake, 1024, 1, fake, 4, 1, 0, 0, fake, 16, None) == -1     # short stride
    assert lib.dq_quantize_pack(h, fake, 1024, 65, fake, 4, 1, 0, 0, fake, 4096, None) == -1  # M too large
    assert lib.dq_unpack_dequant_reduce(h, fake, 4096, 1, fake, 4, None, None) == -1
    assert lib.dq_unpack_dequant_reduce(h, fake, 4100, 1, fake, 4, fake, None) == -1          # stride % 16
    if not plan.has_device:
        assert lib.dq_norm(h, fake, 1024, 1, fake, fake, None) == -2
        assert lib.dq_quantize_pack(h, fake, 1024, 1, fake, 4, 1, 0, 0, fake, 4096, None) == -2
        assert lib.dq_unpack_dequant_reduce(h, fake, 4096, 1, fake, 4, fake, None) == -2
    plan.close()


def test_workload_shapes():
    from paper_2107_14575_amd import workloads as wl
    assert sum(wl.resnet18_cifar10_segments()) == 11_173_962
    assert len(wl.transformer_classifier_segments()) == 102
    seg, g = wl.ragged_mix(M=2)
    starts, dp = wl.seg_starts(seg)
    assert g.shape == (2, dp) and dp % 128 == 0
    valid = np.zeros(dp, dtype=bool)
    for st, n in zip(starts, seg):
        valid[st:st + n] = True
    gn = g.numpy()
    assert np.isnan(gn[:, ~valid]).all() and np.isfinite(gn[:, valid]).all()
    seg2, g2 = wl.ragged_mix(M=2)
    assert np.array_equal(g2.numpy()[:, valid], gn[:, valid])


def test_per_tensor_host_functions_against_the_oracle(dq, oracle):
    rng = np.random.default_rng(7)
    for _ in range(300):
        M, n_seg = int(rng.integers(1, 9)), int(rng.integers(1, 12))
        norms = (10 ** rng.uniform(-6, 1, size=(M, n_seg))).astype(np.float32)
        norms[:, rng.integers(0, n_seg)] = 0
        T = int(rng.integers(1, 500))
        t = int(rng.integers(0, T))
        eps, alpha = float(10 ** rng.uniform(-8, 2)), float(rng.uniform(0.5, 1.0))
        b_min = int(rng.integers(1, 9))
        b_max = int(rng.integers(b_min, 9))
        got_b, got_n = dq.select_bits_per_tensor(norms, t, T, eps, alpha, b_min, b_max)
        want_b, want_n = oracle.select_bits_per_tensor(norms, t, T, eps, alpha, b_min, b_max)
        assert np.array_equal(got_b, want_b)
        assert np.allclose(got_n, want_n, rtol=1e-15, atol=0)
        seg = [int(x) for x in rng.integers(0, 5000, size=n_seg)]
        plan = dq.Plan(seg)
        assert dq.packed_bytes_v(plan, got_b) == oracle.packed_bytes_v(seg, got_b)
        assert dq.comm_cost_bits_per_tensor(M, seg, got_b, 32) == oracle.comm_cost_bits_per_tensor(M, seg, got_b, 32)
        assert dq.packed_bytes_v(plan, [9] * n_seg) == -1
        plan.close()
    with pytest.raises(dq.DQError):
        dq.select_bits_per_tensor(np.ones((2, 2), dtype=np.float32), 5, 5, 0.1, 0.9, 1, 8)


def test_per_worker_rule_against_the_oracle(dq, oracle):
    rng = np.random.default_rng(8)
    for _ in range(500):
        M, n_seg = int(rng.integers(1, 17)), int(rng.integers(1, 10))
        norms = (10 ** rng.uniform(-6, 1, size=(M, n_seg))).astype(np.float32)
        T = int(rng.integers(1, 500))
        t = int(rng.integers(0, T))
        eps, alpha = float(10 ** rng.uniform(-8, 2)), float(rng.uniform(0.5, 1.0))
        b_min = int(rng.integers(1, 9))
        b_max = int(rng.integers(b_min, 9))
        for per_tensor in (False, True):
            got = dq.select_bits_per_worker(norms, t, T, eps, alpha, b_min, b_max, per_tensor=per_tensor)
            want = oracle.select_bits_per_worker(norms, t, T, eps, alpha, b_min, b_max, per_tensor=per_tensor)
            assert np.array_equal(got, want)
    with pytest.raises(dq.DQError):
        dq.select_bits_per_worker(np.ones((2, 2), dtype=np.float32), 0, 5, 0.0, 0.9, 1, 8)


def test_newer_device_entry_points_validate_before_touching_a_gpu(dq):
    """same for the max norm, update, sign-only, one-pass and per-tensor entry points"""
    lib = dq.load_library()
    plan = dq.Plan([1000])           # chunk-local
    wide = dq.Plan([5000])           # not chunk-local
    h, hw = plan.handle, wide.handle
    fake = 0x1000
    assert plan.chunk_local and not wide.chunk_local
    assert lib.dq_plan_is_chunk_local(None) == 0
    assert lib.dq_norm_linf(h, None, 1024, 1, fake, fake, None) == -1
    assert lib.dq_unpack_dequant_reduce_update(h, fake, 4096, 1, fake, 4, 0.1, None, None, None) == -1   # no x
    assert lib.dq_unpack_dequant_reduce_update(h, fake, 4096, 1, fake, 4, float("nan"), fake, None, None) == -1
    assert lib.dq_sign_pack(h, fake, 1024, 1, fake, 112, None) == -1                                   # short stride
    assert lib.dq_sign_reduce(h, fake, 128, 0, None, fake, None) == -1                                 # M < 1
    assert lib.dq_sign_majority(h, fake, 128, 1, None, None) == -1                                     # no output
    assert lib.dq_norm_quantize_pack(hw, fake, 5120, 1, 0, 4, 1, 0, 0, fake, fake, 8192, None) == -1  # not chunk-local
    assert lib.dq_norm_quantize_pack(h, fake, 1024, 1, 0, 9, 1, 0, 0, fake, fake, 8192, None) == -1   # b = 9
    assert lib.dq_quantize_pack_v(h, None, fake, 1024, 1, fake, 1, 0, 0, fake, 8192, None) == -1       # no widths
    assert lib.dq_unpack_dequant_reduce_v(h, None, fake, 8192, 1, fake, fake, None) == -1
    assert lib.dq_select_bits_device(h, None, fake, 1, 0, 5, 0.1, 0.9, 1, 8, 0, None, None, None, None) == -1
    assert lib.dq_widths_set(None, None, None) == -1 and lib.dq_widths_packed_bytes(None) == -1
    lib.dq_widths_destroy(None)      # harmless
    if not plan.has_device:
        import ctypes as C
        w = C.c_void_p()
        assert lib.dq_widths_create(h, C.byref(w)) == -2 and not w.value
        assert lib.dq_norm_linf(h, fake, 1024, 1, fake, fake, None) == -2
        assert lib.dq_sign_pack(h, fake, 1024, 1, fake, 128, None) == -2
        assert lib.dq_sign_reduce(h, fake, 128, 1, None, fake, None) == -2
        assert lib.dq_norm_quantize_pack(h, fake, 1024, 1, 0, 4, 1, 0, 0, fake, fake, 8192, None) == -2
    wide.close()
    plan.close()


def test_rules_agree_with_the_oracle_beyond_one_summation_block(dq, oracle):
    """more than 1024 tensors: the library adds a worker's squared norm block by block, the oracle in
    plain index order (Lemma 1's G-bar_t^2 as written).  Up to 1024 tensors the two orders coincide and
    the results are equal bit for bit; beyond, G-bar agrees to the rounding of a binary64 sum and the
    width is the same unless s* sits within that distance of a level count (either width is then valid)"""
    from tests.pyref import rule_factor, single_width_rule_agrees
    rng = np.random.default_rng(9)
    for n_seg in (1024, 1025, 3000, 70000):
        M = 3
        norms = (10 ** rng.uniform(-4, 0, size=(M, n_seg))).astype(np.float32)
        got = dq.select_bits(norms, 2, 9, 1e-3, 0.9, 1, 8)
        want = oracle.select_bits(norms, 2, 9, 1e-3, 0.9, 1, 8)
        if n_seg <= 1024:
            assert got == want
        assert single_width_rule_agrees(got, want, n_seg, rule_factor(2, 9, 1e-3, 0.9), 1, 8)
        plain = np.sqrt((norms.astype(np.float64) ** 2).sum() / M)
        assert abs(want[1] - plain) <= 1e-13 * plain
        b_got = dq.select_bits_per_worker(norms, 2, 9, 1e-3, 0.9, 1, 8)
        b_want = oracle.select_bits_per_worker(norms, 2, 9, 1e-3, 0.9, 1, 8)
        for i in range(M):
            # a worker's own width (Eq. (17) with its own norm): same validity rule, worker by worker
            n_i = float(np.sqrt((norms[i].astype(np.float64) ** 2).sum()))
            assert len(set(b_got[i])) == 1 and len(set(b_want[i])) == 1
            assert single_width_rule_agrees((b_got[i][0], n_i), (b_want[i][0], n_i), n_seg,
                                            rule_factor(2, 9, 1e-3, 0.9), 1, 8)
