"""Chunk-local plans (no tensor crosses a multiple of 4096 padded elements, e.g. a gradient cut
into buckets): the one-pass norm, and dq_norm_quantize_pack, which reads the gradient once, against
the oracle's norm and quantize+pack."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, _one_step, dq, gpu_norm  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu

LAYOUTS = {
    "granules": [128] * 40,
    "buckets512_ragged_end": [512] * 37,
    "buckets2048": [2048] * 5,
    "buckets4096": [4096] * 3,
    "one_small_tensor": [77],
    "mixed": [4000, 100, 1900, 2048, 77, 0, 3900, 0, 640],
}


def _grads(seg_len, M, seed, scale=1e-2):
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(seed)
    g = torch.full((M, dp), float("nan"), dtype=torch.float32)
    for k, (st, n) in enumerate(zip(starts, seg_len)):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * scale * (1 + k % 5)
    return g


@pytest.mark.parametrize("name", list(LAYOUTS))
def test_two_pass_entry_points_on_chunk_local_plans(dq, oracle, name):
    """dq_norm (now one pass), dq_quantize_pack and the reduce against the oracle, both norms"""
    seg_len = LAYOUTS[name]
    plan = dq.Plan(seg_len)
    assert plan.chunk_local
    plan.close()
    g = _grads(seg_len, 3, 100)
    for b in (1, 4, 7):
        _one_step(dq, oracle, seg_len, g, b, step=b)
    _one_step(dq, oracle, seg_len, g, 3, step=9, linf=True)


@pytest.mark.parametrize("name", list(LAYOUTS))
@pytest.mark.parametrize("linf", [False, True])
def test_one_pass_norm_quantize_pack(dq, oracle, name, linf):
    seg_len = LAYOUTS[name]
    M = 5
    g = _grads(seg_len, M, 101)
    g_host = np.ascontiguousarray(g.numpy())
    g_dev = g.cuda()
    plan = dq.Plan(seg_len)
    two_pass = gpu_norm(dq, plan, g_dev, linf)
    want_norms = (oracle.norm_linf if linf else oracle.norm)(seg_len, g_host)
    for b in range(1, 9):
        nbytes = plan.packed_bytes(b)
        norms = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
        packed = torch.full((M, nbytes + 32), 0xA5, dtype=torch.uint8, device="cuda")
        dq.norm_quantize_pack(plan, g_dev, b, SEED, 40 + b, norms, packed, worker_base=2, linf=linf)
        torch.cuda.synchronize()
        assert torch.equal(norms.view(torch.int32), two_pass.view(torch.int32))     # same values as dq_norm
        n_host = norms.cpu().numpy()
        if linf:
            assert np.array_equal(n_host, want_norms)
        else:
            assert np.all(np.abs(n_host.astype(np.float64) - want_norms) <= np.spacing(want_norms))
        got = packed.cpu().numpy()
        want = oracle.quantize_pack(seg_len, g_host, n_host, b, SEED, 40 + b, worker_base=2)
        assert np.array_equal(got[:, :nbytes], want)
        assert np.all(got[:, nbytes:] == 0xA5)
    plan.close()


def test_bucketed_large_gradient(dq, oracle):
    """D = 2^22 cut into buckets of 512 (8192 tensors), M = 4: norms and messages in full"""
    D, M, b = 1 << 22, 4, 4
    _, g = wl.flat_student_t(D=D, M=M, config=23)
    seg_len = [512] * (D // 512)
    plan = dq.Plan(seg_len)
    g_dev = g.cuda()
    norms = torch.empty((M, plan.n_seg), dtype=torch.float32, device="cuda")
    packed = torch.zeros((M, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    dq.norm_quantize_pack(plan, g_dev, b, SEED, 0, norms, packed)
    torch.cuda.synchronize()
    g_host = np.ascontiguousarray(g.numpy())
    n_host = norms.cpu().numpy()
    want_norms = oracle.norm(seg_len, g_host)
    assert np.all(np.abs(n_host.astype(np.float64) - want_norms) <= np.spacing(want_norms))
    assert np.array_equal(packed.cpu().numpy(), oracle.quantize_pack(seg_len, g_host, n_host, b, SEED, 0))
    # per-bucket norms never exceed the whole-gradient norm and compose to it
    whole = oracle.norm([D], g_host)
    assert np.allclose(np.sqrt((n_host.astype(np.float64) ** 2).sum(axis=1)), whole[:, 0], rtol=1e-6)
    plan.close()


def test_plans_that_are_not_chunk_local_are_refused(dq):
    for seg_len in ([4097], [100, 4096], [2048, 2048, 128, 4096]):
        plan = dq.Plan(seg_len)
        assert not plan.chunk_local
        g = torch.zeros((1, plan.padded_elems), dtype=torch.float32, device="cuda")
        norms = torch.zeros((1, plan.n_seg), dtype=torch.float32, device="cuda")
        packed = torch.zeros((1, plan.packed_bytes(2)), dtype=torch.uint8, device="cuda")
        with pytest.raises(dq.DQError):
            dq.norm_quantize_pack(plan, g, 2, 1, 0, norms, packed)
        plan.close()
    plan = dq.Plan([4096, 2048, 2048])
    assert plan.chunk_local
    plan.close()


def test_algorithm1_lagged_loop_takes_the_single_pass(dq, oracle):
    """the lagged loop on a bucketed plan: single pass and two calls give the same run, bit for bit,
    and every message is the oracle's"""
    from paper_2107_14575_amd import dqsgd
    seg_len = [512] * 9 + [300]
    plan = dq.Plan(seg_len)
    assert plan.chunk_local
    starts, dp = wl.seg_starts(seg_len)
    M, T, eta, alpha, tau, eps_hat = 4, 24, 0.2, 0.9, 4, 0.02
    gen = torch.Generator().manual_seed(102)
    valid = torch.zeros(dp, dtype=torch.bool)
    for st, n in zip(starts, seg_len):
        valid[st:st + n] = True
    target = (torch.randn(dp, generator=gen) * valid).cuda()
    noise = (torch.randn((T, M, dp), generator=gen) * 0.05 * valid).cuda()

    def grad_fn(t, x, grads):
        grads.copy_((x - target).unsqueeze(0) + noise[t])

    seen = []

    def on_step(t, b, grads, norms, packed):
        g_host = np.ascontiguousarray(grads.cpu().numpy())
        want_norms = oracle.norm(seg_len, g_host)
        assert np.all(np.abs(norms.astype(np.float64) - want_norms) <= np.spacing(want_norms))
        assert np.array_equal(packed.cpu().numpy(), oracle.quantize_pack(seg_len, g_host, norms, b, SEED, t))
        seen.append(b)

    x0 = torch.zeros(dp, dtype=torch.float32, device="cuda")
    kw = dict(b0=2, b_min=1, b_max=8, tau=tau, lagged=True, seed=SEED)
    one = dqsgd.run(plan, x0, grad_fn, M, T, eta, eps_hat, alpha, on_step=on_step, **kw)
    two = dqsgd.run(plan, x0, grad_fn, M, T, eta, eps_hat, alpha, one_pass=False, **kw)
    assert one.bits == two.bits == seen and len(set(seen)) >= 3
    assert torch.equal(one.x.view(torch.int32), two.x.view(torch.int32))
    assert one.cost_bits == two.cost_bits
    assert float((one.x - target).norm()) < 0.2 * float(target.norm())
    plan.close()


@pytest.mark.parametrize("name", ["granules", "buckets512_ragged_end", "mixed"])
@pytest.mark.parametrize("linf", [False, True])
def test_one_pass_with_per_tensor_widths(dq, oracle, name, linf):
    seg_len = LAYOUTS[name]
    M = 3
    g = _grads(seg_len, M, 103)
    g_host = np.ascontiguousarray(g.numpy())
    g_dev = g.cuda()
    plan = dq.Plan(seg_len)
    rng = np.random.default_rng(104)
    widths = rng.integers(1, 9, size=len(seg_len)).astype(np.int32)
    table = dq.Widths(plan, widths)
    two_pass = gpu_norm(dq, plan, g_dev, linf)
    norms = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
    packed = torch.full((M, table.packed_bytes + 16), 0xA5, dtype=torch.uint8, device="cuda")
    dq.norm_quantize_pack_v(plan, table, g_dev, SEED, 5, norms, packed, worker_base=1, linf=linf)
    torch.cuda.synchronize()
    assert torch.equal(norms.view(torch.int32), two_pass.view(torch.int32))
    got = packed.cpu().numpy()
    want = oracle.quantize_pack_v(seg_len, g_host, norms.cpu().numpy(), widths, SEED, 5, worker_base=1)
    assert np.array_equal(got[:, :want.shape[1]], want) and np.all(got[:, want.shape[1]:] == 0xA5)
    table.close()
    plan.close()
