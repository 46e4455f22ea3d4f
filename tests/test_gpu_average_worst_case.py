"""Accuracy of the M-way average (Algorithm 1 "Average", Eq. (2)) where it is hardest for binary32
sums: many workers (M = 16, the benchmark's, M = 64, the largest a call accepts, and counts that leave
partial blocks), every term of
one sign so nothing cancels, levels at or near s, norms equal, geometric or spread over four decades.
The messages are written by the oracle from chosen codes; the GPU's average is compared with the
oracle's binary64 one element by element at the benchmark spec's tolerance: 1e-6 of the mean magnitude of
the terms.  The library adds the workers in blocks of eight (an FMA chain per block, then the block
sums), so a value passes through at most 7 + M/8 + 1 roundings: 16 * 2^-24 < 1e-6 at M = 64."""
import numpy as np
import pytest
import torch

from tests.test_gpu_parity import dq  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _norm_sets(M, rng):
    yield "equal", np.full(M, np.float32(1.2345678), dtype=np.float32)
    yield "geometric up", (np.float32(1e-3) * np.float32(1.3) ** np.arange(M)).astype(np.float32)
    yield "geometric down", (np.float32(7.0) * np.float32(0.8) ** np.arange(M)).astype(np.float32)
    yield "four decades", (10.0 ** rng.uniform(-3, 1, size=M)).astype(np.float32)
    yield "one large, rest small", np.concatenate([[np.float32(3.3)], np.full(M - 1, np.float32(1.1e-3))]).astype(np.float32)


@pytest.mark.parametrize("M", [9, 16, 23, 42, 64])   # whole and partial blocks of eight, every load-group tail
@pytest.mark.parametrize("b", [1, 2, 3, 4, 6, 8])
def test_same_sign_terms_near_the_top_level(dq, oracle, M, b):
    rng = np.random.default_rng(1000 * M + b)
    D = 8192 * 3 + 128 * 5          # several reduce tiles and a ragged tail
    seg_len = [D]
    s = (1 << b) - 1
    plan = dq.Plan(seg_len)
    out = torch.empty(D, dtype=torch.float32, device="cuda")
    worst = 0.0
    for negative in (0, 1):
        for name, norms1 in _norm_sets(M, rng):
            norms = norms1.reshape(M, 1)
            # levels: the top level everywhere in the first third, random in the upper half elsewhere
            level = rng.integers(max(1, (s + 1) // 2), s + 1, size=(M, D)).astype(np.uint8)
            level[:, :D // 3] = s
            sign = np.full((M, D), negative, dtype=np.uint8)
            packed = np.stack([oracle.pack(sign[i], level[i], b) for i in range(M)])
            want = oracle.dequant_reduce(seg_len, sign, level, norms, b)
            dq.unpack_dequant_reduce(plan, torch.from_numpy(packed).cuda(), torch.from_numpy(norms).cuda(), b, out)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            unit = (norms / np.float32(s)).astype(np.float32)                       # binary32, as the method defines it
            terms = (level.astype(np.float32) * unit).astype(np.float64)             # each term one binary32 product
            mag = terms.sum(axis=0) / M
            # the oracle's value is the binary64 sum of those terms, divided by M, rounded once
            assert np.array_equal(want, ((-mag if negative else mag)).astype(np.float32)), name
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            assert np.all(err <= 1e-6 * mag), (name, negative, float((err / mag).max()))
            worst = max(worst, float((err / mag).max()))
            # the same messages through a widths table shared by the workers and one with a row per worker
            for table in (dq.Widths(plan, [b]), dq.Widths(plan, [[b]] * M, workers=M)):
                out.fill_(float("nan"))
                dq.unpack_dequant_reduce_v(plan, table, torch.from_numpy(packed).cuda(), torch.from_numpy(norms).cuda(), out)
                torch.cuda.synchronize()
                err_v = np.abs(out.cpu().numpy().astype(np.float64) - want.astype(np.float64))
                assert np.all(err_v <= 1e-6 * mag), (name, negative, "widths table")
                table.close()
    assert worst <= 1e-6
    plan.close()
