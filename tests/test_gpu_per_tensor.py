"""GPU parity for the per-tensor bit-widths: dq_quantize_pack_v, dq_unpack_dequant_reduce_v and
dq_unpack_dequant_reduce_update_v against the oracle's per-tensor functions on the same seeded
inputs -- bitstreams bit for bit, the average within 1e-6 relative."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, _valid_mask, dq, gpu_norm  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _check_average_v(got, want, level, norms, seg_len, widths):
    M = level.shape[0]
    starts, dp = wl.seg_starts(seg_len)
    mag = np.zeros(dp, dtype=np.float64)
    for l, (st, n) in enumerate(zip(starts, seg_len)):
        s = float((1 << int(widths[l])) - 1)
        unit = np.where(norms[:, l] >= np.float32(2.0 ** -100), norms[:, l].astype(np.float64) / s, 0.0)
        mag[st:st + n] = (level[:, st:st + n].astype(np.float64) * unit[:, None]).sum(axis=0) / M
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert err.max() <= 1e-6 * max(np.abs(want).max(), 1e-300)
    assert np.all(err <= 1e-6 * mag + 1.5e-45)
    valid = _valid_mask(seg_len)
    assert np.array_equal(got[~valid].view(np.uint32), np.zeros((~valid).sum(), dtype=np.uint32))


def _one_step_v(dq, oracle, seg_len, grads, widths_list, step, worker_base=0):
    """norm -> quantize+pack -> reduce with per-tensor widths; widths_list holds one or more width
    vectors that are set one after the other on the same table."""
    plan = dq.Plan(seg_len)
    g_host = np.ascontiguousarray(grads.numpy())
    g_dev = grads.cuda()
    M = g_dev.shape[0]
    norms_dev = gpu_norm(dq, plan, g_dev)
    norms = norms_dev.cpu().numpy()
    table = dq.Widths(plan)
    for widths in widths_list:
        widths = np.asarray(widths, dtype=np.int32)
        table.set(widths)
        nbytes = table.packed_bytes
        assert nbytes == oracle.packed_bytes_v(seg_len, widths) == dq.packed_bytes_v(plan, widths)
        packed_dev = torch.full((M, nbytes + 48), 0xA5, dtype=torch.uint8, device="cuda")
        dq.quantize_pack_v(plan, table, g_dev, norms_dev, SEED, step, packed_dev, worker_base=worker_base)
        torch.cuda.synchronize()
        packed = packed_dev.cpu().numpy()
        want_packed = oracle.quantize_pack_v(seg_len, g_host, norms, widths, SEED, step, worker_base)
        assert np.array_equal(packed[:, :nbytes], want_packed)
        assert np.all(packed[:, nbytes:] == 0xA5)
        out = torch.full((plan.padded_elems,), float("nan"), dtype=torch.float32, device="cuda")
        dq.unpack_dequant_reduce_v(plan, table, packed_dev, norms_dev, out)
        torch.cuda.synchronize()
        want_out = oracle.unpack_dequant_reduce_v(seg_len, want_packed, norms, widths)
        _, level = oracle.quantize_v(seg_len, g_host, norms, widths, SEED, step, worker_base)
        _check_average_v(out.cpu().numpy(), want_out, level, norms, seg_len, widths)
    table.close()
    plan.close()
    return norms


def test_ragged_layout_all_widths_at_once(dq, oracle):
    seg_len, grads = wl.ragged_mix(M=3)
    rng = np.random.default_rng(50)
    n = len(seg_len)
    first = np.resize(np.arange(1, 9), n)                      # every width occurs
    second = rng.integers(1, 9, size=n)
    third = first[::-1].copy()
    _one_step_v(dq, oracle, seg_len, grads, [first, second, third], step=5, worker_base=3)


@pytest.mark.parametrize("b", range(1, 9))
def test_equal_widths_reproduce_the_single_width_message(dq, oracle, b):
    seg_len, grads = wl.ragged_mix(M=2)
    plan = dq.Plan(seg_len)
    g_dev = grads.cuda()
    norms_dev = gpu_norm(dq, plan, g_dev)
    table = dq.Widths(plan, [b] * len(seg_len))
    assert table.packed_bytes == plan.packed_bytes(b)
    a = torch.zeros((2, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    c = torch.zeros_like(a)
    dq.quantize_pack(plan, g_dev, norms_dev, b, SEED, 9, a)
    dq.quantize_pack_v(plan, table, g_dev, norms_dev, SEED, 9, c)
    out_a = torch.empty(plan.padded_elems, dtype=torch.float32, device="cuda")
    out_c = torch.empty_like(out_a)
    dq.unpack_dequant_reduce(plan, a, norms_dev, b, out_a)
    dq.unpack_dequant_reduce_v(plan, table, c, norms_dev, out_c)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
    assert torch.equal(out_a.view(torch.int32), out_c.view(torch.int32))
    want = oracle.quantize_pack(seg_len, grads.numpy(), norms_dev.cpu().numpy(), b, SEED, 9)
    assert np.array_equal(c.cpu().numpy(), want)
    table.close()
    plan.close()


def test_width_changes_inside_tiles_waves_and_lane_groups(dq, oracle):
    """one-granule tensors with a different width each: every 128 elements the level stride
    changes, so chunks, waves and workgroup tiles all straddle many widths"""
    rng = np.random.default_rng(51)
    seg_len = [128] * 150 + [100, 28, 1] + [4096 + 256, 128, 8192 + 128, 64]
    widths = rng.integers(1, 9, size=len(seg_len))
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(52)
    g = torch.full((3, dp), float("nan"), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((3, n), generator=gen) * 1e-2
    _one_step_v(dq, oracle, seg_len, g, [widths], step=7)


def test_many_tiny_tensors_with_empty_ones(dq, oracle):
    rng = np.random.default_rng(53)
    seg_len = [int(x) for x in rng.choice([0, 1, 2, 64, 128, 129, 300], size=400)]
    widths = rng.integers(1, 9, size=400)
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(54)
    g = torch.full((2, dp), float("nan"), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((2, n), generator=gen) * 1e-2
    _one_step_v(dq, oracle, seg_len, g, [widths], step=3)


@pytest.mark.parametrize("M", [1, 5, 16])
def test_worker_counts(dq, oracle, M):
    seg_len = [5000, 700, 9000]
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(55 + M)
    g = torch.zeros((M, dp), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * 1e-3
    _one_step_v(dq, oracle, seg_len, g, [[2, 7, 4]], step=2)


def test_resnet18_layout_with_the_rule(dq, oracle):
    """config-2 layout at full size (62 tensors, 11.2 M elements), widths from the per-tensor rule
    applied to the GPU's norms"""
    seg_len, grads = wl.resnet18_like(M=2)
    plan = dq.Plan(seg_len)
    norms = gpu_norm(dq, plan, grads.cuda()).cpu().numpy()
    plan.close()
    T, t, alpha = 100, 60, 0.97
    gbar = float(np.sqrt((norms.astype(np.float64) ** 2).sum() / 2))
    eps_hat = T * alpha ** (T - 1 - t) * (gbar / 100.0) ** 2          # whole-gradient rule lands near b = 7
    widths, nbar = dq.select_bits_per_tensor(norms, t, T, eps_hat, alpha, 1, 8)
    want_widths, want_nbar = oracle.select_bits_per_tensor(norms, t, T, eps_hat, alpha, 1, 8)
    assert np.array_equal(widths, want_widths) and np.allclose(nbar, want_nbar, rtol=1e-15, atol=0)
    b_all, _ = dq.select_bits(norms, t, T, eps_hat, alpha, 1, 8)
    assert np.all(widths <= b_all) and len(set(widths.tolist())) >= 4
    _one_step_v(dq, oracle, seg_len, grads, [widths], step=t)
    # the per-tensor widths send fewer bits than the single width for the same error budget
    assert dq.comm_cost_bits_per_tensor(2, seg_len, widths) < dq.comm_cost_bits(2, int(np.sum(seg_len)), b_all, len(seg_len), 32)
    assert dq.comm_cost_bits_per_tensor(2, seg_len, widths) == oracle.comm_cost_bits_per_tensor(2, seg_len, widths)


def test_update_entry_point(dq, oracle):
    seg_len, grads = wl.ragged_mix(M=4)
    plan = dq.Plan(seg_len)
    dp = plan.padded_elems
    g_dev = grads.cuda()
    norms_dev = gpu_norm(dq, plan, g_dev)
    norms = norms_dev.cpu().numpy()
    widths = np.resize(np.array([3, 1, 8, 5, 2], dtype=np.int32), len(seg_len))
    table = dq.Widths(plan, widths)
    packed = torch.zeros((4, table.packed_bytes), dtype=torch.uint8, device="cuda")
    dq.quantize_pack_v(plan, table, g_dev, norms_dev, SEED, 1, packed)
    rng = np.random.default_rng(56)
    x_init = rng.standard_normal(dp).astype(np.float32)
    valid = _valid_mask(seg_len)
    for with_ghat in (False, True):
        x = torch.from_numpy(x_init.copy()).cuda()
        ghat = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
        dq.unpack_dequant_reduce_update_v(plan, table, packed, norms_dev, 0.37, x, ghat if with_ghat else None)
        torch.cuda.synchronize()
        want_g = oracle.unpack_dequant_reduce_v(seg_len, packed.cpu().numpy(), norms, widths)
        want_x = oracle.update(x_init.copy(), want_g, np.float32(0.37))
        got_x = x.cpu().numpy()
        scale = np.abs(want_g).max()
        assert np.array_equal(got_x[~valid], x_init[~valid])
        assert np.all(np.abs(got_x - want_x) <= 2.0 ** -23 * np.abs(want_x) + 0.37 * 1e-6 * scale)
        if with_ghat:
            np.testing.assert_allclose(ghat.cpu().numpy(), want_g, rtol=0, atol=1e-6 * scale)
    table.close()
    plan.close()


def test_argument_checks(dq):
    seg_len = [300, 0, 50]
    plan = dq.Plan(seg_len)
    other = dq.Plan(seg_len)
    table = dq.Widths(plan)
    g = torch.zeros((1, plan.padded_elems), dtype=torch.float32, device="cuda")
    norms = torch.ones((1, 3), dtype=torch.float32, device="cuda")
    packed = torch.zeros((1, 4096), dtype=torch.uint8, device="cuda")
    out = torch.zeros(plan.padded_elems, dtype=torch.float32, device="cuda")
    assert table.packed_bytes == -1
    with pytest.raises(dq.DQError):                     # widths never set
        dq.quantize_pack_v(plan, table, g, norms, 1, 0, packed)
    for bad in ([0, 1, 1], [1, 9, 1], [1, 1, -3]):
        with pytest.raises(dq.DQError):
            table.set(bad)
    with pytest.raises(ValueError):
        table.set([1, 2])
    table.set([8, 8, 8])
    assert table.packed_bytes == 512 // 8 + 512
    with pytest.raises(dq.DQError):                     # a table made for another plan
        dq.quantize_pack_v(other, table, g, norms, 1, 0, packed)
    short = torch.zeros((1, 512), dtype=torch.uint8, device="cuda")
    with pytest.raises(dq.DQError):                     # stride below the message size
        dq.quantize_pack_v(plan, table, g, norms, 1, 0, short)
    with pytest.raises(dq.DQError):
        dq.unpack_dequant_reduce_v(plan, table, short, norms, out)
    dq.quantize_pack_v(plan, table, g, norms, 1, 0, packed)
    dq.unpack_dequant_reduce_v(plan, table, packed, norms, out)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    table.close()
    other.close()
    plan.close()


def test_algorithm1_loop_with_per_tensor_widths(dq, oracle):
    """Algorithm 1 with one width per tensor on a least-squares problem whose two tensors have very
    different gradient norms: widths, bitstreams, model and cost follow the oracle loop; the
    low-norm tensor is sent with fewer bits than the single-width rule would use."""
    from paper_2107_14575_amd import dqsgd
    seg_len = [700, 300, 77]
    plan = dq.Plan(seg_len)
    starts, dp = wl.seg_starts(seg_len)
    M, T, eta, alpha, tau, eps_hat = 4, 40, 0.2, 0.9, 5, 0.02
    gen = torch.Generator().manual_seed(57)
    target = torch.zeros(dp)
    for (st, n), scale in zip(zip(starts, seg_len), (1.0, 0.01, 0.1)):
        target[st:st + n] = torch.randn(n, generator=gen) * scale
    noise_scale = torch.zeros(dp)
    for (st, n), scale in zip(zip(starts, seg_len), (0.05, 0.0005, 0.005)):
        noise_scale[st:st + n] = scale
    noise = (torch.randn((T, M, dp), generator=gen) * noise_scale).cuda()
    target = target.cuda()

    def grad_fn(t, x, grads):
        grads.copy_((x - target).unsqueeze(0) + noise[t])

    x_or = np.zeros(dp, dtype=np.float32)
    state = dict(b=np.full(3, 2, dtype=np.int32), bits=[], cost=0, single=[])

    def on_step(t, b, grads, norms, packed):
        g_host = np.ascontiguousarray(grads.cpu().numpy())
        assert np.array_equal(b, state["b"]), f"widths differ at t={t}"
        want = oracle.quantize_pack_v(seg_len, g_host, norms, b, SEED, t)
        assert np.array_equal(packed.cpu().numpy(), want), f"bitstream differs at t={t}"
        oracle.update(x_or, oracle.unpack_dequant_reduce_v(seg_len, want, norms, b), eta)
        state["bits"].append(b.copy())
        state["cost"] += oracle.comm_cost_bits_per_tensor(M, seg_len, b, 32)
        if t + 1 < T and (t + 1) % tau == 0:
            state["b"], _ = oracle.select_bits_per_tensor(norms, t + 1, T, eps_hat, alpha, 1, 8)
            state["single"].append(oracle.select_bits(norms, t + 1, T, eps_hat, alpha, 1, 8)[0])

    x0 = torch.zeros(dp, dtype=torch.float32, device="cuda")
    res = dqsgd.run(plan, x0, grad_fn, M, T, eta, eps_hat, alpha, b0=2, b_min=1, b_max=8, tau=tau, lagged=True,
                    seed=SEED, on_step=on_step, per_tensor=True)
    assert all(np.array_equal(a, c) for a, c in zip(res.bits, state["bits"])) and res.cost_bits == state["cost"]
    widths = np.array(res.bits)
    assert len(np.unique(widths)) >= 3 and np.any(widths[:, 0] > widths[:, 1])
    assert all(np.all(state["bits"][tau * (k + 1)] <= s) for k, s in enumerate(state["single"]))
    x_gpu = res.x.cpu().numpy()
    assert np.abs(x_gpu - x_or).max() <= T * (2.0 ** -23 * np.abs(x_or).max() + eta * 1e-6 * 4.0)
    assert float((res.x - target).norm()) < 0.1 * float(target.norm())
    plan.close()
