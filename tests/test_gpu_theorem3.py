"""Algorithm 1 on the GPU against Theorem 3's isotropic case (Eq. (22)) over a whole run.

For F(x) = (lambda/2)||x - x*||^2 and workers that all hold the exact gradient, the only noise is
the quantizer's, and one step obeys E[F(x_{t+1}) - F* | x_t] = beta (F(x_t) - F*) +
(lambda eta^2/2) Tr Sigma(x_t) with beta = (1 - eta*lambda)^2 and Tr Sigma(x_t) =
(1/M^2) sum_i (N_i/s_t)^2 sum_j p_j (1 - p_j) (Appendix A's variance of the rounding).  Unrolled
over T steps, per run r the quantity
    D_r = (F(x_T) - F*) - [ beta^T (F(x_0) - F*) + (lambda eta^2/2) sum_t beta^(T-1-t) Tr Sigma(x_t^r) ]
has mean zero.  The GPU loop is run for many seeds, Tr Sigma is evaluated exactly from each
iteration's gradients, and the mean of D_r is tested against its standard error: pins the update's
sign and step, the 1/M of the average, the level grid and the dynamic widths inside a real run."""
import numpy as np
import pytest
import torch

from paper_2107_14575_amd import workloads as wl
from tests.test_gpu_parity import dq  # noqa: F401  (dq is a fixture)

pytestmark = pytest.mark.gpu


def _trace_sigma(g, N, b, M):
    """exact trace of the covariance of the average of M identical workers' quantized gradients"""
    s = np.float32((1 << b) - 1)
    scale = np.float32(s / np.float32(N))
    a = np.minimum(np.abs(g).astype(np.float32) * scale, s)          # the quantizer's own binary32 steps
    p = (a - np.floor(a)).astype(np.float64)
    unit = float(np.float32(N) / s)
    return unit ** 2 * float((p * (1 - p)).sum()) / M


@pytest.mark.parametrize("rule", ["fixed", "dynamic"])
def test_whole_run_matches_theorem3(dq, rule):
    from paper_2107_14575_amd import dqsgd
    d, M, T, lam, eta, runs = 2048, 4, 25, 0.8, 0.5, 48
    plan = dq.Plan([d])
    dp = plan.padded_elems
    gen = torch.Generator().manual_seed(120)
    x_star = torch.zeros(dp)
    x_star[:d] = torch.randn(d, generator=gen)
    x_star = x_star.cuda()
    x0 = torch.zeros(dp, dtype=torch.float32, device="cuda")
    beta = (1 - eta * lam) ** 2
    F = lambda x: 0.5 * lam * float(((x.double() - x_star.double()) ** 2).sum())

    def grad_fn(t, x, grads):
        grads.copy_((lam * (x - x_star)).unsqueeze(0).expand(M, dp))

    # fixed: b = 2 throughout; dynamic: the lagged rule moves b during the run (norms shrink by
    # sqrt(beta) per step, faster than alpha^(1/2) grows the rule's factor, so b walks down)
    kw = dict(b0=2, b_min=2, b_max=2, tau=1) if rule == "fixed" else dict(b0=6, b_min=1, b_max=8, tau=3)
    eps_hat = T * (float(lam * x_star.norm()) / 40.0) ** 2
    diffs, finals, widths_seen = [], [], set()
    for r in range(runs):
        acc = dict(noise=0.0)

        def on_step(t, b, grads, norms, packed):
            g = grads[0, :d].cpu().numpy()
            acc["noise"] += beta ** (T - 1 - t) * _trace_sigma(g, norms[0, 0], b, M)
            widths_seen.add(b)

        res = dqsgd.run(plan, x0, grad_fn, M, T, eta, eps_hat, 0.9, lagged=True, seed=1000 + r, on_step=on_step, **kw)
        predicted = beta ** T * F(x0) + 0.5 * lam * eta ** 2 * acc["noise"]
        diffs.append(F(res.x) - predicted)
        finals.append(F(res.x))
    diffs = np.array(diffs)
    se = diffs.std(ddof=1) / np.sqrt(runs)
    assert abs(diffs.mean()) <= 5 * se + 1e-6 * np.mean(finals), (diffs.mean(), se)
    # the quantization term matters: without it the prediction would be far off
    assert np.mean(finals) > 3 * beta ** T * F(x0)
    if rule == "dynamic":
        assert len(widths_seen) >= 3
    plan.close()
