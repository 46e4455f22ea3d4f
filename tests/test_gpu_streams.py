"""Streams: the newer entry points enqueue on the stream they are given, and two independent
steps on two streams at once (each with its own plan, widths table and buffers) give the results
of running them one after the other."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, dq  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _make(dq, seg_len, M, seed):
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(seed)
    g = torch.zeros((M, dp), dtype=torch.float32)
    for st, n in zip(starts, seg_len):
        g[:, st:st + n] = torch.randn((M, n), generator=gen) * 1e-2
    plan = dq.Plan(seg_len)
    table = dq.Widths(plan)
    return dict(plan=plan, table=table, g=g.cuda(), M=M,
                norms=torch.zeros((M, plan.n_seg), dtype=torch.float32, device="cuda"),
                ws=torch.zeros(plan.workspace_bytes(M), dtype=torch.uint8, device="cuda"),
                packed=torch.zeros((M, dq.packed_bytes_v(plan, [8] * plan.n_seg)), dtype=torch.uint8, device="cuda"),
                x=torch.zeros(dp, dtype=torch.float32, device="cuda"),
                b=torch.zeros(plan.n_seg, dtype=torch.int32, device="cuda"))


def _step(dq, s, t, stream):
    dq.norm(s["plan"], s["g"], s["norms"], s["ws"], stream=stream)
    dq.select_bits_device(s["plan"], s["table"], s["norms"], t, 20, 1e-3, 0.95, 1, 8, rule="per_tensor", b_out=s["b"],
                          stream=stream)
    dq.quantize_pack_v(s["plan"], s["table"], s["g"], s["norms"], SEED, t, s["packed"], stream=stream)
    dq.unpack_dequant_reduce_update_v(s["plan"], s["table"], s["packed"], s["norms"], 0.1, s["x"], stream=stream)


def test_two_steps_on_two_streams_at_once(dq):
    a = _make(dq, [50000, 300, 0, 90000, 77], 4, 150)
    c = _make(dq, [512] * 200, 6, 151)
    # one after the other on the current stream
    for t in range(3):
        _step(dq, a, t, None)
        _step(dq, c, t, None)
    torch.cuda.synchronize()
    want = [(s["x"].clone(), s["packed"].clone(), s["b"].clone()) for s in (a, c)]
    for s in (a, c):
        s["x"].zero_()
        s["packed"].zero_()
        s["b"].zero_()
    torch.cuda.synchronize()
    sa, sc = torch.cuda.Stream(), torch.cuda.Stream()
    for t in range(3):                                  # interleaved launches, no synchronisation in between
        _step(dq, a, t, sa)
        _step(dq, c, t, sc)
    sa.synchronize()
    sc.synchronize()
    for s, (x, packed, b) in zip((a, c), want):
        assert torch.equal(s["x"].view(torch.int32), x.view(torch.int32))
        assert torch.equal(s["packed"], packed) and torch.equal(s["b"], b)
    for s in (a, c):
        s["table"].close()
        s["plan"].close()


def test_other_entry_points_follow_the_stream_argument(dq):
    s = _make(dq, [512] * 40 + [100], 3, 152)
    plan = s["plan"]
    side = torch.cuda.Stream()
    results = []
    for stream in (None, side):
        norms = torch.zeros_like(s["norms"])
        ninf = torch.zeros_like(s["norms"])
        pk = torch.zeros((3, plan.packed_bytes(4)), dtype=torch.uint8, device="cuda")
        signs = torch.zeros((3, plan.padded_elems // 8), dtype=torch.uint8, device="cuda")
        out = torch.zeros(plan.padded_elems, dtype=torch.float32, device="cuda")
        vote = torch.zeros_like(out)
        torch.cuda.synchronize()
        dq.norm_linf(plan, s["g"], ninf, s["ws"], stream=stream)
        dq.norm_quantize_pack(plan, s["g"], 4, SEED, 1, norms, pk, stream=stream)
        dq.unpack_dequant_reduce(plan, pk, norms, 4, out, stream=stream)
        dq.sign_pack(plan, s["g"], signs, stream=stream)
        dq.sign_majority(plan, signs, vote, stream=stream)
        (side if stream is not None else torch.cuda.current_stream()).synchronize()
        results.append([t.cpu().numpy() for t in (norms, ninf, pk, signs, out, vote)])
    for x, y in zip(*results):
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8))
    s["table"].close()
    plan.close()


def test_bracketed_passes_on_two_streams_with_a_workspace_each(dq):
    """two single-pass calls in flight at once, each with its own workspace, bracket and statistics"""
    cases = [_make(dq, [3 * 4096 + 700, 100, 9000], 3, 153), _make(dq, [20000, 512, 512], 5, 154)]
    for s in cases:
        dq.norm(s["plan"], s["g"], s["norms"], s["ws"])
        s["lo"], s["hi"] = torch.empty_like(s["norms"]), torch.empty_like(s["norms"])
        s["wsb"] = torch.empty(dq.bracketed_workspace_bytes(s["plan"], s["M"]), dtype=torch.uint8, device="cuda")
        s["stats"] = torch.zeros(2, dtype=torch.int64, device="cuda")
        s["n2"] = torch.zeros_like(s["norms"])
        s["pk"] = s["packed"][:, :s["plan"].packed_bytes(3)]
    torch.cuda.synchronize()

    def call(s, t, stream):
        dq.norm_bracket(s["norms"], 0.05, s["lo"], s["hi"], stream=stream)
        dq.norm_quantize_pack_bracketed(s["plan"], s["g"], s["lo"], s["hi"], 3, SEED, t, s["n2"], s["pk"], s["wsb"],
                                        stats=s["stats"], stream=stream)
        dq.unpack_dequant_reduce_update(s["plan"], s["pk"], s["n2"], 3, 0.1, s["x"], stream=stream)

    for t in range(3):
        for s in cases:
            call(s, t, None)
    torch.cuda.synchronize()
    want = [(s["x"].clone(), s["pk"].clone(), s["stats"].clone()) for s in cases]
    for s in cases:
        s["x"].zero_()
        s["packed"].zero_()
        s["stats"].zero_()
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for t in range(3):
        for s, st in zip(cases, streams):
            call(s, t, st)
    for st in streams:
        st.synchronize()
    for s, (x, pk, stats) in zip(cases, want):
        assert torch.equal(s["x"].view(torch.int32), x.view(torch.int32))
        assert torch.equal(s["pk"], pk) and torch.equal(s["stats"], stats)
        assert int(stats[0]) > 0
    for s in cases:
        s["table"].close()
        s["plan"].close()
