"""GPU parity for dq_norm_quantize_pack_bracketed: one pass over the gradient for any layout, given
a bracket for every norm.  Whatever the bracket (tight, wide, wrong, unusable) the norms must be
the l2 norms (1 ulp of the oracle's) and the messages must be the oracle's for those norms, bit for
bit; the statistics say which route the chunks took."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import SEED, dq, gpu_norm  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _run(dq, oracle, seg_len, grads, b, lo_factor, hi_factor, step=3, worker_base=2, check_norm=True, linf=False):
    """-> (exceptions settled, chunks redone, number of (worker, chunk) pairs)"""
    plan = dq.Plan(seg_len)
    M = grads.shape[0]
    g_host = np.ascontiguousarray(grads.numpy())
    g_dev = grads.cuda()
    ref = gpu_norm(dq, plan, g_dev, linf)
    lo = (ref * lo_factor).contiguous()
    hi = (ref * hi_factor).contiguous()
    norms_dev = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = plan.packed_bytes(b)
    packed = torch.full((M, nbytes + 32), 0xA5, dtype=torch.uint8, device="cuda")
    ws = torch.full((dq.bracketed_workspace_bytes(plan, M),), 0xEE, dtype=torch.uint8, device="cuda")  # stale contents
    stats = torch.full((2,), -7, dtype=torch.int64, device="cuda")
    dq.norm_quantize_pack_bracketed(plan, g_dev, lo, hi, b, SEED, step, norms_dev, packed, ws,
                                    worker_base=worker_base, stats=stats, linf=linf)
    torch.cuda.synchronize()
    norms = norms_dev.cpu().numpy()
    if linf:
        assert np.array_equal(norms.view(np.uint32), oracle.norm_linf(seg_len, g_host).view(np.uint32))
    elif check_norm:
        want_n = oracle.norm(seg_len, g_host)
        assert np.all(np.abs(norms.astype(np.float64) - want_n.astype(np.float64)) <= np.spacing(want_n))
    want = oracle.quantize_pack(seg_len, g_host, norms, b, SEED, step, worker_base)
    got = packed.cpu().numpy()
    assert np.array_equal(got[:, :nbytes], want), f"b={b} bracket x[{lo_factor}, {hi_factor}]"
    assert np.all(got[:, nbytes:] == 0xA5)
    n_chunks = (plan.padded_elems + 4095) // 4096
    plan.close()
    s = stats.cpu().numpy()
    assert s[0] >= 0 and 0 <= s[1] <= n_chunks * M
    return int(s[0]), int(s[1]), n_chunks * M


def _flat(D, M, seed, sigma=1e-3):
    gen = torch.Generator().manual_seed(seed)
    return [D], torch.randn((M, (D + 127) // 128 * 128), generator=gen) * sigma


@pytest.mark.parametrize("b", range(1, 9))
def test_flat_gradient_tight_bracket(dq, oracle, b):
    """one tensor over 257 chunks and a ragged tail, bracket +-1 %.  The undecided elements per
    chunk number about 4096 * (hi - lo)/N * E[s|g|/N] (16 at b = 8 for this size): almost every
    chunk is finished by settling its few records, hardly any is quantized twice"""
    seg_len, g = _flat((1 << 20) + 1000, 2, 40 + b)
    settled, redone, total = _run(dq, oracle, seg_len, g, b, 0.99, 1.01)
    assert redone <= total // 50
    assert settled > 0


@pytest.mark.parametrize("b", [1, 2, 5, 8])
def test_flat_gradient_loose_bracket(dq, oracle, b):
    """13 chunks, bracket +-12.5 %: few undecided elements at small b, more than a chunk's 31
    records at large b -- exact either way"""
    seg_len, g = _flat(12 * 4096 + 1000, 3, 60 + b)
    settled, redone, total = _run(dq, oracle, seg_len, g, b, 0.875, 1.125)
    if b <= 2:
        assert redone == 0 and settled > 0
    if b == 8:
        assert redone == total


def test_exact_bracket_settles_nothing(dq, oracle):
    seg_len, g = _flat(5 * 4096, 4, 51)
    # lo = hi = the norm the other kernels compute; the path's own norm may differ from it in the
    # last place, and then every chunk of that worker is redone -- both outcomes are exact
    settled, redone, total = _run(dq, oracle, seg_len, g, 4, 1.0, 1.0)
    assert settled == 0 or redone > 0
    settled, redone, total = _run(dq, oracle, seg_len, g, 4, 1.0 - 2.0 ** -20, 1.0 + 2.0 ** -20)
    assert redone == 0


@pytest.mark.parametrize("factors", [(4.0, 8.0), (0.01, 0.02)])
def test_wrong_bracket_redoes_every_chunk(dq, oracle, factors):
    seg_len, g = _flat(7 * 4096 + 128, 2, 52)
    settled, redone, total = _run(dq, oracle, seg_len, g, 5, *factors)
    assert redone == total and settled == 0


def test_wide_bracket_overflows_some_chunks(dq, oracle):
    """d = 8192 per tensor (two chunks each): a = s|g|/N is large, a bracket of 1/8..8 leaves most
    elements undecided, far more than a chunk's 63 records"""
    seg_len = [8192] * 3
    gen = torch.Generator().manual_seed(53)
    g = torch.randn((3, 3 * 8192), generator=gen)
    settled, redone, total = _run(dq, oracle, seg_len, g, 6, 0.125, 8.0)
    assert redone >= total // 2
    # a mild bracket and few levels on the same data: a handful of undecided elements per chunk
    settled, redone, total = _run(dq, oracle, seg_len, g, 2, 0.99, 1.01)
    assert settled > 0 and redone == 0


def test_tensors_inside_one_chunk_need_no_bracket(dq, oracle):
    """small tensors that do not cross a multiple of 4096: their norms are finished inside the
    kernel, so even a useless bracket (NaN, or wrong by a factor) neither settles nor redoes anything"""
    seg_len = [100, 2000, 0, 1000, 700, 50, 4096, 77, 3000]   # padded: 128 + 2048 + 1024 + 768 + 128 | 4096 | 128 + 3072
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(56)
    g = torch.randn((4, dp), generator=gen) * 1e-2
    g[2, starts[3]:starts[3] + 1000] = 0.0             # a zero tensor: the zero path, decided on the spot
    for factors in ((float("nan"), float("nan")), (5.0, 7.0), (0.9, 1.1)):
        settled, redone, total = _run(dq, oracle, seg_len, g, 5, *factors)
        assert settled == 0 and redone == 0
    # mixed with a tensor that does span chunks: only that one depends on its bracket
    seg_len = [100, 9000, 500]
    starts, dp = wl.seg_starts(seg_len)
    g = torch.randn((2, dp), generator=gen) * 1e-2
    settled, redone, total = _run(dq, oracle, seg_len, g, 3, 0.97, 1.03)
    assert redone == 0
    settled, redone, total = _run(dq, oracle, seg_len, g, 3, 2.0, 3.0)
    assert redone == total                              # every chunk holds a piece of the long tensor


def test_unusable_brackets(dq, oracle):
    """zero tensors (lo = 0), norms below the floor, and a layout with empty tensors"""
    seg_len = [5000, 0, 300, 4096, 77]
    starts, dp = wl.seg_starts(seg_len)
    gen = torch.Generator().manual_seed(54)
    g = torch.randn((3, dp), generator=gen) * 1e-2
    g[:, starts[2]:starts[2] + 300] = 0.0          # a zero tensor
    g[1, starts[3]:starts[3] + 4096] *= 1e-34      # below DQ_MIN_NORM for worker 1
    settled, redone, total = _run(dq, oracle, seg_len, g, 3, 0.9, 1.1)
    assert redone > 0


def test_nan_and_reversed_brackets(dq, oracle):
    seg_len, g = _flat(3 * 4096, 2, 55)
    for lo_f, hi_f in ((float("nan"), 1.1), (0.9, float("nan")), (1.1, 0.9), (0.9, float("inf"))):
        settled, redone, total = _run(dq, oracle, seg_len, g, 4, lo_f, hi_f)
        assert redone == total


@pytest.mark.parametrize("M", [1, 5, 64])
def test_ragged_layout(dq, oracle, M):
    seg_len, g = wl.ragged_mix(M=M)
    for b in (2, 7):
        _run(dq, oracle, seg_len, g, b, 0.8, 1.25, step=b, worker_base=9)
        _run(dq, oracle, seg_len, g, b, 0.8, 1.25, step=b, worker_base=9, linf=True)


@pytest.mark.parametrize("b", [1, 4, 8])
def test_max_norm(dq, oracle, b):
    """p = infinity: norms are exact.  With the max norm s|g|/N is of order s/4, so a +-1 % bracket
    leaves few elements open only for the smallest b; for the others most chunks are done again"""
    seg_len, g = _flat((1 << 18) + 500, 3, 80 + b)
    settled, redone, total = _run(dq, oracle, seg_len, g, b, 0.99, 1.01, linf=True)
    if b == 1:
        assert redone <= total // 10 and settled > 0
    settled, redone, total = _run(dq, oracle, seg_len, g, b, 1.0, 1.0, linf=True)   # maxima are exact: lo = hi = N works
    assert settled == 0 and redone == 0
    settled, redone, total = _run(dq, oracle, seg_len, g, b, 3.0, 4.0, linf=True)
    assert redone == total


def test_heavy_tails_and_sparse_rows(dq, oracle):
    """the value kinds of the benchmark configurations at a size of a few chunks"""
    seg_len, g = wl.flat_student_t(D=1 << 16, M=4, device="cpu")
    settled, redone, total = _run(dq, oracle, seg_len, g, 4, 0.98, 1.02)
    assert redone <= 1 and settled > 0
    seg_len, g = wl.transformer_like(M=2, device="cpu")
    _run(dq, oracle, seg_len, g, 4, 0.875, 1.125)


def test_argument_checks(dq):
    plan = dq.Plan([4096 * 2])
    M = 2
    g = torch.zeros((M, 8192), device="cuda")
    lo = torch.ones((M, 1), device="cuda")
    norms = torch.empty((M, 1), device="cuda")
    packed = torch.empty((M, plan.packed_bytes(4)), dtype=torch.uint8, device="cuda")
    ws = torch.empty(dq.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device="cuda")
    with pytest.raises(dq.DQError):
        dq.norm_quantize_pack_bracketed(plan, g, lo, lo, 9, 1, 0, norms, packed, ws)
    with pytest.raises(dq.DQError):
        short = torch.empty((M, 96), dtype=torch.uint8, device="cuda")
        dq.norm_quantize_pack_bracketed(plan, g, lo, lo, 4, 1, 0, norms, short, ws)
    with pytest.raises(ValueError):
        dq.norm_quantize_pack_bracketed(plan, g, lo, lo, 4, 1, 0, norms, packed, ws[:64])
    assert dq.bracketed_workspace_bytes(plan, 0) == -1
    plan.close()


def test_norm_bracket_helper(dq):
    norms = torch.rand((5, 7), device="cuda") * 3.0
    lo, hi = torch.empty_like(norms), torch.empty_like(norms)
    dq.norm_bracket(norms, 0.125, lo, hi)
    torch.cuda.synchronize()
    assert torch.equal(lo, norms * 0.875) and torch.equal(hi, norms * 1.125)
    for bad in (-0.1, 1.0, float("nan")):
        with pytest.raises(dq.DQError):
            dq.norm_bracket(norms, bad, lo, hi)


@pytest.mark.parametrize("per_worker", [False, True])
def test_per_tensor_widths(dq, oracle, per_worker):
    """the single pass with a widths table: long tensors bracketed, short ones finished in the kernel,
    widths 1..8 mixed; tight, loose and wrong brackets give the oracle's messages for the call's norms"""
    seg_len = [9000, 100, 3 * 4096 + 700, 0, 2000, 40000, 77]
    starts, dp = wl.seg_starts(seg_len)
    M = 3
    gen = torch.Generator().manual_seed(57)
    g = torch.randn((M, dp), generator=gen) * 1e-2
    g_host = np.ascontiguousarray(g.numpy())
    g_dev = g.cuda()
    plan = dq.Plan(seg_len)
    rng = np.random.default_rng(58)
    widths = rng.integers(1, 9, size=(M, len(seg_len)) if per_worker else len(seg_len)).astype(np.int32)
    table = dq.Widths(plan, widths, workers=M if per_worker else None)
    ref = gpu_norm(dq, plan, g_dev)
    wsb = torch.empty(dq.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device="cuda")
    stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    seen = []
    for lo_f, hi_f in ((0.99, 1.01), (0.7, 1.4), (2.0, 3.0), (float("nan"), 1.0)):
        norms_dev = torch.full((M, plan.n_seg), float("nan"), dtype=torch.float32, device="cuda")
        packed = torch.zeros((M, table.packed_bytes + 16), dtype=torch.uint8, device="cuda")
        packed[:, table.packed_bytes:] = 0xA5
        dq.norm_quantize_pack_bracketed_v(plan, table, g_dev, (ref * lo_f).contiguous(), (ref * hi_f).contiguous(), SEED, 4,
                                          norms_dev, packed, wsb, worker_base=1, stats=stats)
        torch.cuda.synchronize()
        norms = norms_dev.cpu().numpy()
        want_n = oracle.norm(seg_len, g_host)
        assert np.all(np.abs(norms.astype(np.float64) - want_n.astype(np.float64)) <= np.spacing(want_n))
        got = packed.cpu().numpy()
        if per_worker:
            want = oracle.quantize_pack_w(seg_len, g_host, norms, widths, SEED, 4, 1)
            for i in range(M):
                n = table.worker_packed_bytes(i)
                assert np.array_equal(got[i, :n], want[i, :n]), (lo_f, i)
                assert np.all(got[i, n:table.packed_bytes] == 0)
        else:
            want = oracle.quantize_pack_v(seg_len, g_host, norms, widths, SEED, 4, 1)
            assert np.array_equal(got[:, :table.packed_bytes], want), lo_f
        assert np.all(got[:, table.packed_bytes:] == 0xA5)
        seen.append(stats.cpu().numpy().copy())
    assert seen[0][0] > 0                                  # a tight bracket settles a few elements afterwards
    assert seen[2][1] > 0 and seen[3][1] > 0               # a wrong or unusable one sends chunks through the redo map
    table.close()
    plan.close()


def test_between_the_two_settle_forms(dq):
    """81920 (worker, chunk) pairs: past the 2^16 limit of the wavefront-per-chunk settle kernel, so the
    lane-per-chunk kernel and the map-walking redo kernel run on a plan far smaller than the
    full-size one.  Compared with the two calls on the device (themselves checked against the oracle)."""
    D, M, b = (1 << 26) + 4096 * 3 + 500, 5, 3
    seg_len, g = wl.flat_student_t(D=D, M=M, device="cuda")
    plan = dq.Plan(seg_len)
    assert M * ((plan.padded_elems + 4095) // 4096) > (1 << 16)
    ref = gpu_norm(dq, plan, g)
    wsb = torch.empty(dq.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device="cuda")
    stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    norms = torch.empty_like(ref)
    packed = torch.empty((M, plan.packed_bytes(b)), dtype=torch.uint8, device="cuda")
    want = torch.empty_like(packed)
    for lo_f, hi_f, all_again in ((0.95, 1.05, False), (1.5, 2.0, True)):
        packed.fill_(0x3C)
        dq.norm_quantize_pack_bracketed(plan, g, (ref * lo_f).contiguous(), (ref * hi_f).contiguous(), b, SEED, 6, norms,
                                        packed, wsb, stats=stats)
        dq.quantize_pack(plan, g, norms, b, SEED, 6, want)
        torch.cuda.synchronize()
        assert float(((norms.double() - ref.double()).abs() / ref.double()).max()) <= 2.0 ** -23
        assert torch.equal(packed, want)
        n_pairs = M * ((plan.padded_elems + 4095) // 4096)
        assert (int(stats[1]) == n_pairs) if all_again else (int(stats[1]) == 0 and int(stats[0]) > 0)
    plan.close()
