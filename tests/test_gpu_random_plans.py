"""GPU parity on seeded random layouts: tensor lists (empty, tiny, ragged, several tiles long),
worker counts, strides wider than the padded gradient, value kinds (Gaussian at any scale, heavy
tails, mostly zero, one-hot, all zero, below the norm floor, signed zeros), widths, seeds, steps
and worker numbers are all drawn from a generator seeded by the case number.  Pads and the slack
behind each worker's gradient hold NaN and huge values: nothing may depend on them.  Every entry
point family is compared with the oracle: widths and messages bit for bit, averages to 1e-6."""
import numpy as np
import pytest
import torch

from tests.test_gpu_parity import dq  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

KINDS = ("gauss", "t3", "sparse", "onehot", "zeros", "tiny", "signed_zeros")


def _lengths(rng, chunk_local):
    if chunk_local:
        # tensors of 1..4096 elements laid out so that none crosses a multiple of 4096 padded elements
        lens, pos = [], 0
        for _ in range(int(rng.integers(1, 60))):
            room = 4096 - pos % 4096
            n = int(rng.choice([0, 1, 100, 128, 129, 512, 1000, 2048, 4096]))
            if (n + 127) // 128 * 128 > room:
                n = int(rng.integers(max(room - 127, 1), room + 1))  # fills the chunk exactly
            lens.append(n)
            pos += (n + 127) // 128 * 128
        return lens
    n_seg = int(rng.integers(1, 40))
    pick = lambda: int(rng.choice([0, int(rng.integers(1, 10)), int(rng.integers(120, 140)),
                                   int(rng.integers(1, 5000)), int(rng.integers(5000, 30000))],
                                  p=[0.1, 0.2, 0.2, 0.4, 0.1]))
    lens = [pick() for _ in range(n_seg)]
    if sum(lens) == 0:
        lens[0] = 77
    return lens


def _gradients(rng, seg_len, M):
    starts, pos = [], 0
    for n in seg_len:
        starts.append(pos)
        pos += (n + 127) // 128 * 128
    dp = pos
    stride = dp + 4 * int(rng.integers(0, 40))
    g = np.empty((M, stride), dtype=np.float32)
    g[:, 0::2] = np.nan          # pads and slack: poison
    g[:, 1::2] = 3.0e38
    for st, n in zip(starts, seg_len):
        if n == 0:
            continue
        kind = KINDS[int(rng.integers(0, len(KINDS)))]
        sigma = 10.0 ** rng.uniform(-6, 2)
        if kind == "gauss":
            v = rng.standard_normal((M, n)) * sigma
        elif kind == "t3":
            v = rng.standard_t(3, size=(M, n)) * sigma
        elif kind == "sparse":
            v = rng.standard_normal((M, n)) * sigma * (rng.random((M, n)) < 0.1)
        elif kind == "onehot":
            v = np.zeros((M, n))
            v[np.arange(M), rng.integers(0, n, size=M)] = sigma * rng.choice([-1.0, 1.0], size=M)
        elif kind == "zeros":
            v = np.zeros((M, n))
        elif kind == "tiny":
            v = rng.standard_normal((M, n)) * 1e-36   # norms below 2^-100: the zero path
        else:
            v = np.where(rng.random((M, n)) < 0.5, -0.0, 0.0) + (rng.random((M, n)) < 0.2) * sigma
        g[:, st:st + n] = v.astype(np.float32)
    return starts, dp, g


def _valid(starts, seg_len, dp):
    m = np.zeros(dp, dtype=bool)
    for st, n in zip(starts, seg_len):
        m[st:st + n] = True
    return m


def _check_average(got, want, per_worker_terms, valid):
    """overall 1e-6 of the largest value; per element 1e-6 of the mean magnitude of the M terms
    (plus one binary32 denormal); pads exactly +0"""
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert err.max() <= 1e-6 * max(np.abs(want).max(), 1e-300)
    mag = np.mean(np.abs(np.stack(per_worker_terms).astype(np.float64)), axis=0)
    assert np.all(err <= 1e-6 * mag + 1.5e-45)
    assert np.array_equal(got[~valid].view(np.uint32), np.zeros((~valid).sum(), dtype=np.uint32))


@pytest.mark.parametrize("case", range(60))
def test_random_layout(dq, oracle, case):
    rng = np.random.default_rng(90000 + case)
    chunk_local = case % 3 == 2
    seg_len = _lengths(rng, chunk_local)
    M = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 33, 64]))
    starts, dp, g_host = _gradients(rng, seg_len, M)
    n_seg = len(seg_len)
    b = int(rng.integers(1, 9))
    seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
    step = int(rng.integers(0, 2 ** 32))
    worker_base = int(rng.integers(0, 2 ** 32 - M))
    linf = bool(rng.integers(0, 2))
    print(f"case {case}: n_seg={n_seg} D'={dp} M={M} b={b} linf={linf} chunk_local={chunk_local}", flush=True)

    plan = dq.Plan(seg_len)
    assert plan.padded_elems == dp and plan.chunk_local == (chunk_local or plan.chunk_local)
    valid = _valid(starts, seg_len, dp)
    g_dev = torch.from_numpy(g_host).cuda()
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device="cuda")
    norms_dev = torch.full((M, n_seg), float("nan"), dtype=torch.float32, device="cuda")
    (dq.norm_linf if linf else dq.norm)(plan, g_dev, norms_dev, ws)
    torch.cuda.synchronize()
    norms = norms_dev.cpu().numpy()
    if linf:
        assert np.array_equal(norms.view(np.uint32), oracle.norm_linf(seg_len, g_host).view(np.uint32))
    else:
        want_n = oracle.norm(seg_len, g_host)
        assert np.all(np.abs(norms.astype(np.float64) - want_n.astype(np.float64)) <= np.spacing(want_n))

    # ---- the bit rules on the device against the oracle's (Eq. (17); single width, per tensor)
    T = int(rng.integers(1, 400))
    t = int(rng.integers(0, T))
    alpha = float(rng.uniform(0.5, 1.0))
    gbar = float(np.sqrt((norms.astype(np.float64) ** 2).sum() / M)) if not linf else \
        float(np.sqrt((norms.astype(np.float64).max(axis=1) ** 2).sum() / M))
    eps_hat = max(T * (gbar / float(rng.uniform(0.5, 300.0))) ** 2 * alpha ** (T - 1 - t), 1e-200)  # s* in 0.5..300
    rule_table = dq.Widths(plan)
    b_dev = torch.full((n_seg,), -1, dtype=torch.int32, device="cuda")
    bytes_dev = torch.zeros(1, dtype=torch.int64, device="cuda")
    for rule in ("single_linf" if linf else "single", "per_tensor"):
        dq.select_bits_device(plan, rule_table, norms_dev, t, T, eps_hat, alpha, 1, 8, rule=rule, b_out=b_dev,
                              packed_bytes_out=bytes_dev)
        torch.cuda.synchronize()
        if rule == "per_tensor":
            want_b, _ = oracle.select_bits_per_tensor(norms, t, T, eps_hat, alpha, 1, 8)
        else:
            one, _ = (oracle.select_bits_linf if linf else oracle.select_bits)(norms, t, T, eps_hat, alpha, 1, 8)
            want_b = np.full(n_seg, one, dtype=np.int32)
        assert np.array_equal(b_dev.cpu().numpy(), want_b), rule
        assert int(bytes_dev[0]) == oracle.packed_bytes_v(seg_len, want_b)
    rule_table.close()

    # ---- one width for everything
    nbytes = plan.packed_bytes(b)
    slack = 16 * int(rng.integers(0, 4))
    packed = torch.full((M, nbytes + slack), 0xA5, dtype=torch.uint8, device="cuda")
    dq.quantize_pack(plan, g_dev, norms_dev, b, seed, step, packed, worker_base=worker_base)
    out = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
    dq.unpack_dequant_reduce(plan, packed, norms_dev, b, out)
    torch.cuda.synchronize()
    want_pk = oracle.quantize_pack(seg_len, g_host, norms, b, seed, step, worker_base)
    got_pk = packed.cpu().numpy()
    assert np.array_equal(got_pk[:, :nbytes], want_pk)
    assert np.all(got_pk[:, nbytes:] == 0xA5)
    want_out = oracle.unpack_dequant_reduce(seg_len, want_pk, norms, b)
    terms = [oracle.unpack_dequant_reduce(seg_len, want_pk[i:i + 1], norms[i:i + 1], b) for i in range(M)]
    _check_average(out.cpu().numpy(), want_out, terms, valid)

    # ---- the same step in one pass over the gradient where the layout allows it
    if plan.chunk_local:
        n2 = torch.full((M, n_seg), float("nan"), dtype=torch.float32, device="cuda")
        pk2 = torch.full_like(packed, 0xA5)
        dq.norm_quantize_pack(plan, g_dev, b, seed, step, n2, pk2, worker_base=worker_base, linf=linf)
        torch.cuda.synchronize()
        assert torch.equal(n2.view(torch.int32), norms_dev.view(torch.int32))
        assert torch.equal(pk2, packed)

    # ---- norms and messages in one pass given a bracket for every norm: any bracket must give the
    # messages of the two-pass route for the norms the call computes
    margin = float(rng.choice([0.0, 1e-3, 0.05, 0.5]))
    lo_dev, hi_dev = norms_dev * (1.0 - margin), norms_dev * (1.0 + margin)
    if case % 5 == 0:
        lo_dev, hi_dev = norms_dev * 2.0, norms_dev * 3.0        # wrong: every chunk with a long tensor is done again
    n3 = torch.full((M, n_seg), float("nan"), dtype=torch.float32, device="cuda")
    pk3 = torch.full_like(packed, 0xA5)
    wsb = torch.full((dq.bracketed_workspace_bytes(plan, M),), 0x5A, dtype=torch.uint8, device="cuda")
    dq.norm_quantize_pack_bracketed(plan, g_dev, lo_dev, hi_dev, b, seed, step, n3, pk3, wsb,
                                    worker_base=worker_base, linf=linf)
    torch.cuda.synchronize()
    n3_host = n3.cpu().numpy()
    if linf:
        assert np.array_equal(n3_host.view(np.uint32), norms.view(np.uint32))
    else:
        assert np.all(np.abs(n3_host.astype(np.float64) - want_n.astype(np.float64)) <= np.spacing(want_n))
    got3 = pk3.cpu().numpy()
    assert np.array_equal(got3[:, :nbytes], oracle.quantize_pack(seg_len, g_host, n3_host, b, seed, step, worker_base))
    assert np.all(got3[:, nbytes:] == 0xA5)

    # ---- one width per tensor
    b_seg = rng.integers(1, 9, size=n_seg).astype(np.int32)
    table = dq.Widths(plan, b_seg)
    assert table.packed_bytes == oracle.packed_bytes_v(seg_len, b_seg)
    pk_v = torch.full((M, table.packed_bytes + slack), 0xA5, dtype=torch.uint8, device="cuda")
    dq.quantize_pack_v(plan, table, g_dev, norms_dev, seed, step, pk_v, worker_base=worker_base)
    out_v = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
    dq.unpack_dequant_reduce_v(plan, table, pk_v, norms_dev, out_v)
    torch.cuda.synchronize()
    want_v = oracle.quantize_pack_v(seg_len, g_host, norms, b_seg, seed, step, worker_base)
    got_v = pk_v.cpu().numpy()
    assert np.array_equal(got_v[:, :table.packed_bytes], want_v)
    assert np.all(got_v[:, table.packed_bytes:] == 0xA5)
    # the same messages from the single pass with bracketed norms (any bracket)
    pk_bv = torch.full_like(pk_v, 0xA5)
    n_bv = torch.full((M, n_seg), float("nan"), dtype=torch.float32, device="cuda")
    dq.norm_quantize_pack_bracketed_v(plan, table, g_dev, lo_dev, hi_dev, seed, step, n_bv, pk_bv, wsb,
                                      worker_base=worker_base, linf=linf)
    torch.cuda.synchronize()
    assert torch.equal(n_bv.view(torch.int32), n3.view(torch.int32))
    assert np.array_equal(pk_bv.cpu().numpy()[:, :table.packed_bytes],
                          oracle.quantize_pack_v(seg_len, g_host, n3_host, b_seg, seed, step, worker_base))
    assert np.all(pk_bv.cpu().numpy()[:, table.packed_bytes:] == 0xA5)
    want_out_v = oracle.unpack_dequant_reduce_v(seg_len, want_v, norms, b_seg)
    terms = [oracle.unpack_dequant_reduce_v(seg_len, want_v[i:i + 1], norms[i:i + 1], b_seg) for i in range(M)]
    _check_average(out_v.cpu().numpy(), want_out_v, terms, valid)
    table.close()

    # ---- one width per worker and tensor
    b_w = rng.integers(1, 9, size=(M, n_seg)).astype(np.int32)
    table = dq.Widths(plan, b_w, workers=M)
    pk_w = torch.zeros((M, table.packed_bytes), dtype=torch.uint8, device="cuda")
    dq.quantize_pack_v(plan, table, g_dev, norms_dev, seed, step, pk_w, worker_base=worker_base)
    out_w = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
    dq.unpack_dequant_reduce_v(plan, table, pk_w, norms_dev, out_w)
    torch.cuda.synchronize()
    want_w = oracle.quantize_pack_w(seg_len, g_host, norms, b_w, seed, step, worker_base)
    got_w = pk_w.cpu().numpy()
    for i in range(M):
        n = table.worker_packed_bytes(i)
        assert n == oracle.packed_bytes_v(seg_len, b_w[i])
        assert np.array_equal(got_w[i, :n], want_w[i, :n]), i
        assert np.all(got_w[i, n:] == 0)
    pk_bw = torch.zeros_like(pk_w)
    dq.norm_quantize_pack_bracketed_v(plan, table, g_dev, lo_dev, hi_dev, seed, step, n_bv, pk_bw, wsb,
                                      worker_base=worker_base, linf=linf)
    torch.cuda.synchronize()
    want_bw = oracle.quantize_pack_w(seg_len, g_host, n3_host, b_w, seed, step, worker_base)
    got_bw = pk_bw.cpu().numpy()
    for i in range(M):
        n = table.worker_packed_bytes(i)
        assert np.array_equal(got_bw[i, :n], want_bw[i, :n]), i
        assert np.all(got_bw[i, n:] == 0)
    want_out_w = oracle.unpack_dequant_reduce_w(seg_len, want_w, norms, b_w)
    terms = [oracle.unpack_dequant_reduce_v(seg_len, want_w[i:i + 1, :oracle.packed_bytes_v(seg_len, b_w[i])],
                                            norms[i:i + 1], b_w[i]) for i in range(M)]
    _check_average(out_w.cpu().numpy(), want_out_w, terms, valid)
    table.close()

    # ---- sign-only messages: mean of signs, scaled mean, majority vote
    sp = torch.full((M, dp // 8 + slack), 0xA5, dtype=torch.uint8, device="cuda")
    dq.sign_pack(plan, g_dev, sp)
    torch.cuda.synchronize()
    want_sp = oracle.sign_pack(seg_len, g_host)
    got_sp = sp.cpu().numpy()
    assert np.array_equal(got_sp[:, :dp // 8], want_sp)
    assert np.all(got_sp[:, dp // 8:] == 0xA5)
    assert np.array_equal(got_sp[:, :dp // 8], got_pk[:, :dp // 8])   # the sign plane of the full message
    scales = np.abs(rng.standard_normal((M, n_seg))).astype(np.float32)
    scales_dev = torch.from_numpy(scales).cuda()
    o = torch.full((dp,), float("nan"), dtype=torch.float32, device="cuda")
    dq.sign_reduce(plan, sp, o)
    torch.cuda.synchronize()
    want_mean = oracle.sign_reduce(seg_len, want_sp)
    got_mean = o.cpu().numpy()
    assert np.abs(got_mean.astype(np.float64) - want_mean).max() <= 1e-6                   # values in [-1, 1]
    assert np.array_equal(got_mean[~valid].view(np.uint32), np.zeros((~valid).sum(), dtype=np.uint32))
    dq.sign_majority(plan, sp, o)
    torch.cuda.synchronize()
    assert np.array_equal(o.cpu().numpy(), oracle.sign_reduce(seg_len, want_sp, majority=True))
    dq.sign_reduce(plan, sp, o, scales=scales_dev)
    torch.cuda.synchronize()
    want_s = oracle.sign_reduce(seg_len, want_sp, scales=scales)
    terms = [oracle.sign_reduce(seg_len, want_sp[i:i + 1], scales=scales[i:i + 1]) for i in range(M)]
    _check_average(o.cpu().numpy(), want_s, terms, valid)
    plan.close()
