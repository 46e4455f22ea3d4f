"""GPU parity where a padded index no longer fits 32 bits: one worker with 2^34 + 12588 elements
(64 GiB of fp32).  Byte offsets into the gradient pass 2^33 at element 2^31, element indices pass
2^32, the sign plane's byte offsets pass 2^31 and the Philox counter's second word becomes 1 at
element 2^34.  Windows around each of those places and the ragged tail are compared with the
oracle bit for bit; whole buffers are compared between entry points on the device."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl

pytestmark = pytest.mark.gpu

SEED = wl.QUANT_SEED
D = (1 << 34) + 3 * 4096 + 300  # last granule: 44 valid elements, 84 pads
DP = (D + 127) // 128 * 128
WORKER, STEP = 7, 9


@pytest.fixture(scope="module")
def dq():
    import paper_2107_14575_amd as dq
    dq.load_library()
    assert torch.cuda.is_available()
    return dq


@pytest.fixture(scope="module")
def big(dq):
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    need = DP * 4 * 3 + DP * 9 // 8 + (6 << 30)  # gradient, two averages, one b = 8 message, tables
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of device memory, {free >> 30} GiB are free")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260)
    g = torch.empty((1, DP), dtype=torch.float32, device="cuda")
    for c0 in range(0, DP, 1 << 28):
        piece = g[0, c0:c0 + (1 << 28)]
        piece.normal_(generator=gen)
        piece.mul_(1e-3)
    plan = dq.Plan([D])
    norms = torch.empty((1, 1), dtype=torch.float32, device="cuda")
    ws = torch.empty(plan.workspace_bytes(1), dtype=torch.uint8, device="cuda")
    dq.norm(plan, g, norms, ws)
    torch.cuda.synchronize()
    yield g, plan, norms, ws
    plan.close()
    del g
    torch.cuda.empty_cache()


WINDOWS = [(0, 4096), ((1 << 31) - 4096, (1 << 31) + 4096), ((1 << 32) - 4096, (1 << 32) + 4096),
           ((1 << 34) - 8192, (1 << 34) + 8192), (DP - 8192, DP)]


def test_plan_and_norms(dq, big):
    g, plan, norms, ws = big
    assert plan.padded_elems == DP
    total = 0.0
    top = 0.0
    for c0 in range(0, D, 1 << 27):
        piece = g[0, c0:min(c0 + (1 << 27), D)]
        total += float((piece.double() ** 2).sum())
        top = max(top, float(piece.abs().max()))
    want = np.float32(np.sqrt(total))
    assert abs(float(norms[0, 0]) - float(want)) <= np.spacing(want)
    n_inf = torch.empty_like(norms)
    dq.norm_linf(plan, g, n_inf, ws)
    torch.cuda.synchronize()
    assert float(n_inf[0, 0]) == top


@pytest.mark.parametrize("b", [3, 8])
def test_codes_and_average_in_windows(dq, oracle, big, b):
    g, plan, norms_dev, _ = big
    norms = norms_dev.cpu().numpy()
    pk = torch.empty((1, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    out = torch.empty(DP, dtype=torch.float32, device="cuda")
    dq.quantize_pack(plan, g, norms_dev, b, SEED, STEP, pk, worker_base=WORKER)
    dq.unpack_dequant_reduce(plan, pk, norms_dev, b, out)
    torch.cuda.synchronize()
    for p0, p1 in WINDOWS:
        g_slice = np.ascontiguousarray(g[:, p0:p1].cpu().numpy())
        sign, level = oracle.quantize_range([D], g_slice, norms, b, SEED, STEP, p0, p1, worker_base=WORKER)
        want = oracle.pack(sign[0], level[0], b)
        n = p1 - p0
        lv0 = DP // 8 + p0 // 8 * b
        assert np.array_equal(pk[0, p0 // 8:p1 // 8].cpu().numpy(), want[:n // 8]), (b, p0)
        assert np.array_equal(pk[0, lv0:lv0 + n // 8 * b].cpu().numpy(), want[n // 8:]), (b, p0)
        want_out = oracle.dequant_reduce_range([D], sign, level, norms, b, p0, p1)
        assert np.array_equal(out[p0:p1].cpu().numpy(), want_out), (b, p0)  # M = 1: one product, exact
    # what lies past the tensor's end is zero bits and +0
    assert int(pk[0, D // 8 + 1:DP // 8].max()) == 0
    assert int(pk[0, DP // 8 + (D + 7) // 8 * b:].max()) == 0
    assert float(out[D:].abs().max()) == 0.0
    # |Q(g)_j - g_j| <= N/s at every element
    bound = float(norms[0, 0]) / ((1 << b) - 1) * (1 + 2.0 ** -20)
    worst = 0.0
    for c0 in range(0, D, 1 << 27):
        c1 = min(c0 + (1 << 27), D)
        worst = max(worst, float((out[c0:c1] - g[0, c0:c1]).abs().max()))
    assert worst <= bound
    # the other entry points on the same input give the same bytes and the same average
    sp = torch.empty((1, DP // 8), dtype=torch.uint8, device="cuda")
    dq.sign_pack(plan, g, sp)
    torch.cuda.synchronize()
    assert torch.equal(sp[0], pk[0, :DP // 8])
    del sp
    # one pass with a bracket: records and fix-ups past index 2^32, partial-sum slots past 2^22 chunks
    wsb = torch.empty(dq.bracketed_workspace_bytes(plan, 1), dtype=torch.uint8, device="cuda")
    pk_b = torch.empty_like(pk)
    norms_b = torch.empty_like(norms_dev)
    stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    dq.norm_quantize_pack_bracketed(plan, g, norms_dev * 0.9, norms_dev * 1.1, b, SEED, STEP, norms_b, pk_b, wsb,
                                    worker_base=WORKER, stats=stats)
    torch.cuda.synchronize()
    if torch.equal(norms_b, norms_dev):
        assert torch.equal(pk_b, pk)
    else:
        assert abs(float(norms_b[0, 0]) - float(norms_dev[0, 0])) <= np.spacing(np.float32(norms_dev[0, 0].item()))
        dq.quantize_pack(plan, g, norms_b, b, SEED, STEP, pk, worker_base=WORKER)
        torch.cuda.synchronize()
        assert torch.equal(pk_b, pk)
        dq.quantize_pack(plan, g, norms_dev, b, SEED, STEP, pk, worker_base=WORKER)
        torch.cuda.synchronize()
    assert int(stats[0]) > 0
    del pk_b, wsb
    torch.cuda.empty_cache()
    table = dq.Widths(plan, [b])
    pk_v = torch.empty_like(pk)
    dq.quantize_pack_v(plan, table, g, norms_dev, SEED, STEP, pk_v, worker_base=WORKER)
    torch.cuda.synchronize()
    assert torch.equal(pk_v, pk)
    del pk_v
    torch.cuda.empty_cache()
    out_v = torch.empty_like(out)
    dq.unpack_dequant_reduce_v(plan, table, pk, norms_dev, out_v)
    torch.cuda.synchronize()
    assert torch.equal(out_v, out)
    table.close()
    del out_v, out, pk
    torch.cuda.empty_cache()
