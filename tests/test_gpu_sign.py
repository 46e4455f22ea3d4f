"""GPU parity for the sign-only baseline: dq_sign_pack bit for bit, dq_sign_majority exactly,
dq_sign_reduce within 1e-6 of the mean scale, against the oracle."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import _valid_mask, dq  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _sign_step(dq, oracle, seg_len, grads, scales=None):
    plan = dq.Plan(seg_len)
    dp = plan.padded_elems
    M = grads.shape[0]
    g_dev = grads.cuda()
    packed = torch.full((M, dp // 8 + 32), 0xA5, dtype=torch.uint8, device="cuda")
    dq.sign_pack(plan, g_dev, packed)
    torch.cuda.synchronize()
    got = packed.cpu().numpy()
    want = oracle.sign_pack(seg_len, np.ascontiguousarray(grads.numpy()))
    assert np.array_equal(got[:, :dp // 8], want)
    assert np.all(got[:, dp // 8:] == 0xA5)
    valid = _valid_mask(seg_len)
    zeros = np.zeros((~valid).sum(), dtype=np.uint32)

    out = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
    dq.sign_majority(plan, packed, out)
    torch.cuda.synchronize()
    vote = out.cpu().numpy()
    assert np.array_equal(vote, oracle.sign_reduce(seg_len, want, majority=True))
    assert np.array_equal(vote[~valid].view(np.uint32), zeros)

    for sc in (None, scales):
        out.fill_(float("nan"))
        dq.sign_reduce(plan, packed, out, scales=None if sc is None else torch.from_numpy(sc).cuda())
        torch.cuda.synchronize()
        mean = out.cpu().numpy()
        want_mean = oracle.sign_reduce(seg_len, want, scales=sc)
        bound = 1e-6 * (1.0 if sc is None else float(np.abs(sc).mean(axis=0).max()))
        assert np.abs(mean.astype(np.float64) - want_mean).max() <= bound
        assert np.array_equal(mean[~valid].view(np.uint32), zeros)
    plan.close()


@pytest.mark.parametrize("M", [1, 2, 7, 8, 16, 64])
def test_ragged_layout(dq, oracle, M):
    seg_len, grads = wl.ragged_mix(M=M)
    rng = np.random.default_rng(70 + M)
    scales = rng.uniform(0.01, 3.0, size=(M, len(seg_len))).astype(np.float32)
    _sign_step(dq, oracle, seg_len, grads, scales)


@pytest.mark.parametrize("D", [1, 127, 128, 8192, 8192 + 128, 8192 * 5 + 77])
def test_tile_boundaries(dq, oracle, D):
    seg_len, grads = wl.flat_gaussian(D=D, M=3, config=71)
    scales = np.array([[0.5], [2.0], [1.25]], dtype=np.float32)
    _sign_step(dq, oracle, seg_len, grads, scales)


def test_many_tiny_tensors_zeros_and_negative_zeros(dq, oracle):
    rng = np.random.default_rng(72)
    seg_len = [int(x) for x in rng.choice([0, 1, 2, 64, 128, 129, 300], size=300)]
    starts, dp = wl.seg_starts(seg_len)
    g = torch.full((4, dp), float("nan"), dtype=torch.float32)
    g = -g.abs()                                                  # pads: NaN with the sign bit set
    gen = torch.Generator().manual_seed(73)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((4, n), generator=gen)
        if n > 1:
            g[0, st] = 0.0
            g[1, st] = -0.0
    scales = rng.uniform(0.1, 1.0, size=(4, len(seg_len))).astype(np.float32)
    _sign_step(dq, oracle, seg_len, g, scales)


def test_transformer_layout_full_size(dq, oracle):
    seg_len, grads = wl.transformer_like(M=4)
    _sign_step(dq, oracle, seg_len, grads, None)


def test_argument_checks(dq):
    plan = dq.Plan([1000])
    g = torch.zeros((2, plan.padded_elems), dtype=torch.float32, device="cuda")
    out = torch.zeros(plan.padded_elems, dtype=torch.float32, device="cuda")
    short = torch.zeros((2, 112), dtype=torch.uint8, device="cuda")     # message needs 128 bytes
    with pytest.raises(dq.DQError):
        dq.sign_pack(plan, g, short)
    with pytest.raises(dq.DQError):
        dq.sign_reduce(plan, short, out)
    with pytest.raises(dq.DQError):
        dq.sign_majority(plan, short, out)
    plan.close()
