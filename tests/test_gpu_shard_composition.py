"""The server side of a sharded deployment, shown on one GPU: G ranks each quantize their whole
gradient; rank k receives from every rank the sign bytes and the level bytes of shard k (two
contiguous pieces of the sender's message) and reduces them with a plan that describes the shard's
pieces of tensors, the parent tensors' norms beside them.  The result must be the matching slice
of the unsharded reduce, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, dq, gpu_norm  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu

TILE = 8192   # shards are cut at multiples of the reduce tile


def _shard_plan(seg_len, p0, p1):
    """tensor pieces inside padded range [p0, p1): (lengths, parent index of each piece)"""
    starts, _ = wl.seg_starts(seg_len)
    lens, parents = [], []
    for l, (st, n) in enumerate(zip(starts, seg_len)):
        pad = -(-n // 128) * 128
        lo, hi = max(st, p0), min(st + pad, p1)
        if lo >= hi:
            continue
        valid = max(0, min(st + n, hi) - lo)
        # a piece keeps its padded extent inside the shard: valid elements first, pads after
        assert (hi - lo) % 128 == 0
        lens.append((valid, hi - lo))
        parents.append(l)
    return lens, parents


@pytest.mark.parametrize("b", [1, 4, 7])
def test_shard_reduce_equals_the_slice_of_the_full_reduce(dq, b):
    G = 4
    seg_len = [20000, 5, 0, 9000, 40000, 130, 16384 + 77]
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(140)
    g = torch.zeros((G, dp), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((G, n), generator=gen) * 1e-2
    plan = dq.Plan(seg_len)
    g_dev = g.cuda()
    norms = gpu_norm(dq, plan, g_dev)
    packed = torch.zeros((G, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    dq.quantize_pack(plan, g_dev, norms, b, SEED, 3, packed)          # every rank's own worker side
    full = torch.empty(dp, dtype=torch.float32, device="cuda")
    dq.unpack_dequant_reduce(plan, packed, norms, b, full)
    torch.cuda.synchronize()

    n_tiles = -(-dp // TILE)
    per = -(-n_tiles // G)
    covered = 0
    for k in range(G):
        p0, p1 = min(k * per * TILE, dp), min((k + 1) * per * TILE, dp)
        if p0 >= p1:
            continue
        pieces, parents = _shard_plan(seg_len, p0, p1)
        # cuts fall at multiples of 128 inside a tensor or at a tensor's padded end, so every piece
        # is again a tensor of a plan: `valid` elements followed by the pads up to `extent`
        lens = []
        for valid, extent in pieces:
            assert -(-valid // 128) * 128 == extent, (valid, extent)
            lens.append(valid)
        shard = dq.Plan(lens)
        assert shard.padded_elems == p1 - p0
        shard_norms = norms[:, parents].contiguous()                   # the parents' norms travel with the shard
        # what rank k receives from rank i: two contiguous pieces of i's message
        sign = packed[:, p0 // 8:p1 // 8]
        level = packed[:, dp // 8 + p0 * b // 8: dp // 8 + p1 * b // 8]
        recv = torch.cat([sign, level], dim=1).contiguous()
        assert recv.shape[1] == shard.packed_bytes(b)
        out = torch.empty(p1 - p0, dtype=torch.float32, device="cuda")
        dq.unpack_dequant_reduce(shard, recv, shard_norms, b, out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), full[p0:p1].view(torch.int32)), k
        covered += p1 - p0
        shard.close()
    assert covered == dp
    plan.close()


def test_rank_by_rank_worker_side_equals_the_simulated_workers(dq):
    """rank i quantizing its own gradient with worker_base = i produces row i of the M-worker call
    (the Philox counter carries the global worker id), also through the one-pass kernel"""
    seg_len = [512] * 30 + [100]
    starts, dp = wl.seg_starts(seg_len)
    M, b = 5, 3
    gen = torch.Generator().manual_seed(141)
    g = torch.zeros((M, dp), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * 1e-2
    plan = dq.Plan(seg_len)
    g_dev = g.cuda()
    norms = gpu_norm(dq, plan, g_dev)
    together = torch.zeros((M, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    dq.quantize_pack(plan, g_dev, norms, b, SEED, 9, together)
    for i in range(M):
        alone = torch.zeros((1, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
        dq.quantize_pack(plan, g_dev[i:i + 1], norms[i:i + 1], b, SEED, 9, alone, worker_base=i)
        fused = torch.zeros_like(alone)
        n_out = torch.empty((1, plan.n_seg), dtype=torch.float32, device="cuda")
        dq.norm_quantize_pack(plan, g_dev[i:i + 1], b, SEED, 9, n_out, fused, worker_base=i)
        torch.cuda.synchronize()
        assert torch.equal(alone[0], together[i]) and torch.equal(fused[0], together[i])
        assert torch.equal(n_out.view(torch.int32), norms[i:i + 1].view(torch.int32))
    plan.close()
