"""GPU parity for per-worker (and per-worker-per-tensor) bit-widths: the *_v entry points with a
widths table that has one row per worker, against the oracle's per-worker functions."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, _valid_mask, dq, gpu_norm  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _step_w(dq, oracle, seg_len, grads, widths, step, worker_base=0, one_pass=False):
    plan = dq.Plan(seg_len)
    M = grads.shape[0]
    g_host = np.ascontiguousarray(grads.numpy())
    g_dev = grads.cuda()
    widths = np.asarray(widths, dtype=np.int32).reshape(M, len(seg_len))
    table = dq.Widths(plan, widths, workers=M)
    assert table.packed_bytes == max(oracle.packed_bytes_v(seg_len, widths[i]) for i in range(M))
    for i in range(M):
        assert table.worker_packed_bytes(i) == oracle.packed_bytes_v(seg_len, widths[i])
    packed = torch.zeros((M, table.packed_bytes + 32), dtype=torch.uint8, device="cuda")
    packed[:, table.packed_bytes:] = 0xA5
    if one_pass:
        norms_dev = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
        dq.norm_quantize_pack_v(plan, table, g_dev, SEED, step, norms_dev, packed, worker_base=worker_base)
        assert torch.equal(norms_dev.view(torch.int32), gpu_norm(dq, plan, g_dev).view(torch.int32))
    else:
        norms_dev = gpu_norm(dq, plan, g_dev)
        dq.quantize_pack_v(plan, table, g_dev, norms_dev, SEED, step, packed, worker_base=worker_base)
    torch.cuda.synchronize()
    norms = norms_dev.cpu().numpy()
    want = oracle.quantize_pack_w(seg_len, g_host, norms, widths, SEED, step, worker_base)
    got = packed.cpu().numpy()
    for i in range(M):          # a shorter message leaves the rest of its slot untouched (zeros here)
        n = table.worker_packed_bytes(i)
        assert np.array_equal(got[i, :n], want[i, :n]), i
        assert np.all(got[i, n:table.packed_bytes] == 0)
    assert np.all(got[:, table.packed_bytes:] == 0xA5)
    out = torch.full((plan.padded_elems,), float("nan"), dtype=torch.float32, device="cuda")
    dq.unpack_dequant_reduce_v(plan, table, packed, norms_dev, out)
    torch.cuda.synchronize()
    want_out = oracle.unpack_dequant_reduce_w(seg_len, want, norms, widths)
    res = out.cpu().numpy()
    valid = _valid_mask(seg_len)
    err = np.abs(res.astype(np.float64) - want_out)
    assert err.max() <= 1e-6 * max(np.abs(want_out).max(), 1e-300)
    assert np.array_equal(res[~valid].view(np.uint32), np.zeros((~valid).sum(), dtype=np.uint32))
    # fused update with the same table
    rng = np.random.default_rng(5)
    x_init = rng.standard_normal(plan.padded_elems).astype(np.float32)
    x = torch.from_numpy(x_init.copy()).cuda()
    dq.unpack_dequant_reduce_update_v(plan, table, packed, norms_dev, 0.25, x)
    torch.cuda.synchronize()
    want_x = oracle.update(x_init.copy(), want_out, np.float32(0.25))
    got_x = x.cpu().numpy()
    assert np.array_equal(got_x[~valid], x_init[~valid])
    assert np.all(np.abs(got_x - want_x) <= 2.0 ** -23 * np.abs(want_x) + 0.25 * 1e-6 * np.abs(want_out).max())
    table.close()
    plan.close()


@pytest.mark.parametrize("M", [1, 3, 8, 16, 33, 64])   # beyond 32 workers the reduce's table needs more than 64 KiB of LDS
def test_ragged_layout_random_widths(dq, oracle, M):
    seg_len, grads = wl.ragged_mix(M=M)
    rng = np.random.default_rng(130 + M)
    widths = rng.integers(1, 9, size=(M, len(seg_len)))
    _step_w(dq, oracle, seg_len, grads, widths, step=M, worker_base=1)


def test_one_width_per_worker_from_the_rule(dq, oracle):
    """workers whose gradients differ in scale by 30x: the rule gives them different widths"""
    seg_len = [5000, 700, 0, 9000]
    starts, dp = wl.seg_starts(seg_len)
    M = 6
    gen = torch.Generator().manual_seed(131)
    g = torch.zeros((M, dp), dtype=torch.float32)
    for i in range(M):
        for st, n in zip(starts, seg_len):
            g[i, st:st + n] = torch.randn(n, generator=gen) * (1e-3 * 2.0 ** i)
    plan = dq.Plan(seg_len)
    norms = gpu_norm(dq, plan, g.cuda()).cpu().numpy()
    plan.close()
    T, t, alpha = 50, 30, 0.95
    whole = np.sqrt((norms.astype(np.float64) ** 2).sum(axis=1))
    eps = T * alpha ** (T - 1 - t) * (whole[2] / 10.0) ** 2
    for per_tensor in (False, True):
        widths = dq.select_bits_per_worker(norms, t, T, eps, alpha, 1, 8, per_tensor=per_tensor)
        assert np.array_equal(widths, oracle.select_bits_per_worker(norms, t, T, eps, alpha, 1, 8, per_tensor=per_tensor))
        assert len(np.unique(widths[:, 0])) >= 4 and np.all(np.diff(widths[:, 0]) >= 0)
        if not per_tensor:
            assert np.all(widths == widths[:, :1])
        _step_w(dq, oracle, seg_len, g, widths, step=t)


def test_equal_rows_reproduce_the_shared_table(dq, oracle):
    seg_len, grads = wl.ragged_mix(M=4)
    plan = dq.Plan(seg_len)
    g_dev = grads.cuda()
    norms_dev = gpu_norm(dq, plan, g_dev)
    row = np.resize(np.arange(1, 9, dtype=np.int32), len(seg_len))
    shared = dq.Widths(plan, row)
    per_worker = dq.Widths(plan, np.tile(row, (4, 1)), workers=4)
    a = torch.zeros((4, shared.packed_bytes), dtype=torch.uint8, device="cuda")
    c = torch.zeros_like(a)
    dq.quantize_pack_v(plan, shared, g_dev, norms_dev, SEED, 3, a)
    dq.quantize_pack_v(plan, per_worker, g_dev, norms_dev, SEED, 3, c)
    oa = torch.empty(plan.padded_elems, dtype=torch.float32, device="cuda")
    oc = torch.empty_like(oa)
    dq.unpack_dequant_reduce_v(plan, shared, a, norms_dev, oa)
    dq.unpack_dequant_reduce_v(plan, per_worker, c, norms_dev, oc)
    torch.cuda.synchronize()
    assert torch.equal(a, c) and torch.equal(oa.view(torch.int32), oc.view(torch.int32))
    shared.close()
    per_worker.close()
    plan.close()


def test_one_pass_on_a_chunk_local_plan(dq, oracle):
    seg_len = [512] * 9 + [300, 100, 0, 2048]
    starts, dp = wl.seg_starts(seg_len)
    M = 3
    gen = torch.Generator().manual_seed(132)
    g = torch.full((M, dp), float("nan"), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * 1e-2
    rng = np.random.default_rng(133)
    _step_w(dq, oracle, seg_len, g, rng.integers(1, 9, size=(M, len(seg_len))), step=2, one_pass=True)


def test_argument_checks(dq):
    plan = dq.Plan([300, 50])
    table = dq.Widths(plan, [[1, 2], [3, 4]], workers=2)
    g = torch.zeros((3, plan.padded_elems), dtype=torch.float32, device="cuda")
    norms = torch.ones((3, 2), dtype=torch.float32, device="cuda")
    packed = torch.zeros((3, 4096), dtype=torch.uint8, device="cuda")
    out = torch.zeros(plan.padded_elems, dtype=torch.float32, device="cuda")
    with pytest.raises(dq.DQError):                      # table has 2 rows, call has 3 workers
        dq.quantize_pack_v(plan, table, g, norms, 1, 0, packed)
    with pytest.raises(dq.DQError):
        dq.unpack_dequant_reduce_v(plan, table, packed, norms, out)
    with pytest.raises(dq.DQError):                      # the device rules fill shared tables only
        dq.select_bits_device(plan, table, norms[:2], 0, 5, 0.1, 0.9, 1, 8)
    with pytest.raises(ValueError):
        table.set([1, 2])
    with pytest.raises(dq.DQError):
        dq.Widths(plan, workers=0)
    assert table.worker_packed_bytes(2) == -1
    dq.quantize_pack_v(plan, table, g[:2], norms[:2], 1, 0, packed[:2])
    dq.unpack_dequant_reduce_v(plan, table, packed[:2], norms[:2], out)
    torch.cuda.synchronize()
    table.close()
    plan.close()


@pytest.mark.parametrize("per_tensor", [False, True])
def test_algorithm1_loop_with_per_worker_widths(dq, oracle, per_tensor):
    """workers whose noise differs by 8x each step: every worker picks its own width; widths,
    bitstreams and the model follow the oracle loop"""
    from paper_2107_14575_amd import dqsgd
    seg_len = [700, 300, 77]
    plan = dq.Plan(seg_len)
    starts, dp = wl.seg_starts(seg_len)
    M, T, eta, alpha, tau, eps_hat = 4, 30, 0.2, 0.9, 5, 0.05
    gen = torch.Generator().manual_seed(134)
    valid = torch.zeros(dp)
    for st, n in zip(starts, seg_len):
        valid[st:st + n] = 1
    target = (torch.randn(dp, generator=gen) * valid).cuda()
    scale = torch.tensor([0.02, 0.05, 0.1, 0.16]).view(1, M, 1)
    noise = (torch.randn((T, M, dp), generator=gen) * scale * valid).cuda()

    def grad_fn(t, x, grads):
        grads.copy_((x - target).unsqueeze(0) + noise[t])

    x_or = np.zeros(dp, dtype=np.float32)
    state = dict(b=np.full((M, 3), 2, dtype=np.int32), bits=[])

    def on_step(t, b, grads, norms, packed):
        g_host = np.ascontiguousarray(grads.cpu().numpy())
        assert np.array_equal(b, state["b"]), t
        want = oracle.quantize_pack_w(seg_len, g_host, norms, b, SEED, t)
        got = packed.cpu().numpy()
        for i in range(M):
            n = oracle.packed_bytes_v(seg_len, b[i])
            assert np.array_equal(got[i, :n], want[i, :n]), (t, i)
        oracle.update(x_or, oracle.unpack_dequant_reduce_w(seg_len, want, norms, b), eta)
        state["bits"].append(b.copy())
        if t + 1 < T and (t + 1) % tau == 0:
            state["b"] = oracle.select_bits_per_worker(norms, t + 1, T, eps_hat, alpha, 1, 8, per_tensor=per_tensor)

    x0 = torch.zeros(dp, dtype=torch.float32, device="cuda")
    res = dqsgd.run(plan, x0, grad_fn, M, T, eta, eps_hat, alpha, b0=2, b_min=1, b_max=8, tau=tau, lagged=True,
                    seed=SEED, on_step=on_step, per_worker=True, per_tensor=per_tensor)
    assert all(np.array_equal(a, c) for a, c in zip(res.bits, state["bits"]))
    last = res.bits[-1]
    assert len(np.unique(last[:, 0])) >= 2                       # the workers really differ
    x_gpu = res.x.cpu().numpy()
    assert np.abs(x_gpu - x_or).max() <= T * (2.0 ** -23 * np.abs(x_or).max() + eta * 1e-6 * 4.0)
    assert float((res.x - target).norm()) < 0.2 * float(target.norm())
    plan.close()
