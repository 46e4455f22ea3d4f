"""The device entry points only enqueue kernels on the stream they are given (no allocation, no
memset, no synchronisation), so a step can be captured into a HIP graph and replayed.  The graph
is replayed several times with eager work and synchronisations in between, and every replay is
compared with the same calls made eagerly."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, dq  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _setup(dq, seg_len, M, seed):
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(seed)
    g = torch.zeros((M, dp), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * 1e-2
    plan = dq.Plan(seg_len)
    bufs = dict(
        g=g.cuda(), norms=torch.zeros((M, plan.n_seg), dtype=torch.float32, device="cuda"),
        ws=torch.zeros(plan.workspace_bytes(M), dtype=torch.uint8, device="cuda"),
        packed=torch.zeros((M, dq.packed_bytes_v(plan, [8] * plan.n_seg)), dtype=torch.uint8, device="cuda"),
        x=torch.zeros(dp, dtype=torch.float32, device="cuda"),
        b=torch.zeros(plan.n_seg, dtype=torch.int32, device="cuda"))
    return plan, bufs


def test_device_rule_step_in_a_graph(dq):
    seg_len = [5000, 300, 0, 9000, 77]
    M, T, t, eps, alpha, eta = 4, 50, 20, 1e-3, 0.95, 0.1
    plan, B = _setup(dq, seg_len, M, 110)
    table = dq.Widths(plan)

    def step():
        dq.norm(plan, B["g"], B["norms"], B["ws"])
        dq.select_bits_device(plan, table, B["norms"], t, T, eps, alpha, 1, 8, rule="per_tensor", b_out=B["b"])
        dq.quantize_pack_v(plan, table, B["g"], B["norms"], SEED, t, B["packed"])
        dq.unpack_dequant_reduce_update_v(plan, table, B["packed"], B["norms"], eta, B["x"])

    # eager: three steps, remembering x after each
    want = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        want.append(B["x"].clone())
    want_b = B["b"].clone()

    B["x"].zero_()
    B["b"].zero_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    B["x"].zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(B["x"].view(torch.int32), want[k].view(torch.int32)), f"replay {k}"
        assert torch.equal(B["b"], want_b)
        # eager work of the program's own between the replays
        scratch = torch.empty_like(B["norms"])
        dq.norm_linf(plan, B["g"], scratch, B["ws"])
        assert float(scratch.sum()) > 0
        torch.cuda.synchronize()
    table.close()
    plan.close()


def test_one_pass_lagged_step_in_a_graph(dq):
    seg_len = [512] * 20 + [100]
    M, b, eta = 3, 3, 0.05
    plan, B = _setup(dq, seg_len, M, 111)
    assert plan.chunk_local
    pk = B["packed"][:, :plan.packed_bytes(b)]

    def step():
        dq.norm_quantize_pack(plan, B["g"], b, SEED, 7, B["norms"], pk)
        dq.unpack_dequant_reduce_update(plan, pk, B["norms"], b, eta, B["x"])

    want = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        want.append(B["x"].clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    B["x"].zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(B["x"].view(torch.int32), want[k].view(torch.int32)), f"replay {k}"
        dq.norm(plan, B["g"], torch.empty_like(B["norms"]), B["ws"])
        torch.cuda.synchronize()
    plan.close()


def test_bracketed_step_in_a_graph(dq):
    """norms and messages in one pass with a bracket from the previous norms, then the fused update;
    the statistics counters are part of the graph (a zeroing kernel, no memset)"""
    seg_len = [3 * 4096 + 700, 100, 9000]
    M, b, eta = 3, 3, 0.05
    plan, B = _setup(dq, seg_len, M, 112)
    pk = B["packed"][:, :plan.packed_bytes(b)]
    dq.norm(plan, B["g"], B["norms"], B["ws"])
    torch.cuda.synchronize()
    lo, hi = B["norms"] * 0.9, B["norms"] * 1.1
    wsb = torch.empty(dq.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device="cuda")
    stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    norms2 = torch.empty_like(B["norms"])

    def step():
        dq.norm_quantize_pack_bracketed(plan, B["g"], lo, hi, b, SEED, 7, norms2, pk, wsb, stats=stats)
        dq.unpack_dequant_reduce_update(plan, pk, norms2, b, eta, B["x"])

    want = []
    for _ in range(3):
        step()
        torch.cuda.synchronize()
        want.append(B["x"].clone())
    want_stats = stats.clone()
    assert int(want_stats[0]) > 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    B["x"].zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(3):
        stats.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(B["x"].view(torch.int32), want[k].view(torch.int32)), f"replay {k}"
        assert torch.equal(stats, want_stats)
        dq.norm(plan, B["g"], torch.empty_like(B["norms"]), B["ws"])
        torch.cuda.synchronize()
    plan.close()
