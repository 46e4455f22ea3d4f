"""dq_norm_static_scratch -- the norm pass for callers that cannot allocate (its partial sums live in a
fixed device array inside the library) -- against dq_norm / dq_norm_linf with a caller's workspace:
the same kernels, so the same norms bit for bit; also within 1 ulp of the oracle's norm of Eq. (5).
Two calls in a row on one GPU, the second on a smaller input, share the one array."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dq():
    import paper_2107_14575_amd as dq
    dq.load_library()
    return dq


def _both(dq, seg_len, grads_dev, linf):
    plan = dq.Plan(seg_len)
    M = grads_dev.shape[0]
    assert plan.workspace_bytes(M) <= dq.norm_static_scratch_max_bytes()
    want = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device="cuda")
    (dq.norm_linf if linf else dq.norm)(plan, grads_dev, want, ws)
    before = torch.cuda.memory_allocated()
    dq.norm_static_scratch(plan, grads_dev, got, linf=linf)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    plan.close()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("linf", [False, True])
def test_two_calls_in_a_row_the_second_smaller(dq, oracle, linf):
    gen = torch.Generator().manual_seed(5150)
    # first call: tensors of many 4096-element pieces (multi-item sums through the scratch), ragged tails, M = 8
    seg_big = [300000, 4097, 0, 77, 4096, 123457, 9000]
    _, dp_big = wl.seg_starts(seg_big)
    g_big = torch.randn((8, dp_big), generator=gen) * 1e-2
    got, want = _both(dq, seg_big, g_big.cuda(), linf)
    assert np.array_equal(got, want)
    orc = (oracle.norm_linf if linf else oracle.norm)(seg_big, np.ascontiguousarray(g_big.numpy()))
    assert np.all(np.abs(got.astype(np.float64) - orc.astype(np.float64)) <= (0 if linf else np.spacing(orc)))
    # second call: smaller layout, fewer workers; whatever the first call left in the array must not matter
    seg_small = [9000, 5, 20000]
    _, dp_small = wl.seg_starts(seg_small)
    g_small = torch.randn((3, dp_small), generator=gen) * 3.0
    got, want = _both(dq, seg_small, g_small.cuda(), linf)
    assert np.array_equal(got, want)
    orc = (oracle.norm_linf if linf else oracle.norm)(seg_small, np.ascontiguousarray(g_small.numpy()))
    assert np.all(np.abs(got.astype(np.float64) - orc.astype(np.float64)) <= (0 if linf else np.spacing(orc)))


def test_limit_is_enforced(dq):
    """one piece more than the array holds: a clear error and nothing enqueued"""
    n_items = dq.norm_static_scratch_max_bytes() // 8 // 2 + 1          # M = 2 workers
    plan = dq.Plan([n_items * 4096])
    assert plan.workspace_bytes(2) > dq.norm_static_scratch_max_bytes()
    fake_g = torch.empty(16, dtype=torch.float32, device="cuda")       # never touched: the call is refused first
    out = torch.full((2, 1), -1.0, dtype=torch.float32, device="cuda")
    with pytest.raises(dq.DQError) as err:
        load = dq.load_library()
        status = load.dq_norm_static_scratch(plan.handle, fake_g.data_ptr(), plan.padded_elems, 2, 0, out.data_ptr(), None)
        if status != 0:
            raise dq.DQError("dq_norm_static_scratch", status, load.dq_status_string(status).decode())
    assert err.value.status == -1
    torch.cuda.synchronize()
    assert float(out.min()) == -1.0
    plan.close()
