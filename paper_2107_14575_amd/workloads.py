"""Seeded synthetic gradients shaped like the paper's workloads.

Only shapes, value distributions and sparsity structure live here -- none of the quantizer's
arithmetic -- so the tests can feed the same bytes to the GPU library and to the CPU oracle.  The
paper's datasets and trained models (CIFAR-10/ResNet-18, AG-News text classifier) are not
available; these inputs stand in for their gradients.

Layout: every generator returns ``(seg_len, grads)`` with ``grads`` a float32 torch tensor
``[M][D']`` in the padded layout of ``include/dq.h`` (each tensor padded to a multiple of 128
elements).  Pad elements are filled with ``pad_value`` (NaN by default: the library must ignore
them).  Data seed = 1000*config + worker.
"""
from __future__ import annotations

import math

import numpy as np
import torch

GRANULE = 128
QUANT_SEED = 0xD05C6D  # the quantizer's Philox key used by tests and bench


def padded(n: int) -> int:
    return (n + GRANULE - 1) // GRANULE * GRANULE


def seg_starts(seg_len):
    starts, p = [], 0
    for n in seg_len:
        starts.append(p)
        p += padded(int(n))
    return starts, p


# ------------------------------------------------------------------------------------------ shapes
def resnet18_cifar10_segments():
    """The 62 parameter tensors of the 10-class CIFAR ResNet-18: 11,173,962 parameters."""
    segs = [64 * 3 * 3 * 3, 64, 64]  # stem conv + BN weight, bias
    c_in = 64
    for c in (64, 128, 256, 512):
        for block in range(2):
            first = block == 0
            segs += [c * (c_in if first else c) * 9, c, c]  # conv a + BN
            segs += [c * c * 9, c, c]                        # conv b + BN
            if first and c != 64:
                segs += [c * c_in, c, c]                     # 1x1 downsample conv + BN
        c_in = c
    segs += [10 * 512, 10]
    assert len(segs) == 62 and sum(segs) == 11_173_962
    return segs


def transformer_classifier_segments():
    """Token embedding 30000x256, positions 512x256, 6 layers (d_model 256, ffn 1024), final
    LayerNorm and a 4-class head: 102 tensors, 12,551,172 parameters."""
    d, ffn = 256, 1024
    segs = [30000 * d, 512 * d]
    for _ in range(6):
        segs += [d * d, d] * 4          # q, k, v, o projections with biases
        segs += [d, d, d, d]            # two LayerNorms
        segs += [ffn * d, ffn, d * ffn, d]
    segs += [d, d, 4 * d, 4]
    assert len(segs) == 102 and sum(segs) == 12_551_172
    return segs


# ------------------------------------------------------------------------------------ distributions
def _gen(seed: int, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(n, gen, device):
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32)


def _laplace(n, gen, device):
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float32) - 0.5
    return -torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.4999999))


def _student_t3(n, gen, device):
    z = _normal(n, gen, device)
    chi = _normal(n, gen, device).square_()
    chi += _normal(n, gen, device).square_()
    chi += _normal(n, gen, device).square_()
    return z.div_(chi.div_(3.0).sqrt_().clamp_(min=1e-20))


def _alloc(seg_len, M, device, pad_value):
    _, dp = seg_starts(seg_len)
    grads = torch.full((M, dp), float(pad_value), dtype=torch.float32, device=device)
    return grads


# ------------------------------------------------------------------------------------------ configs
def flat_gaussian(D=1 << 20, M=4, sigma=1e-3, config=1, device="cpu", pad_value=float("nan")):
    """Config 1: one tensor, i.i.d. N(0, sigma^2); worker i from data seed 1000*config + i."""
    seg_len = [D]
    grads = _alloc(seg_len, M, device, pad_value)
    for i in range(M):
        grads[i, :D] = _normal(D, _gen(1000 * config + i, device), device) * sigma
    return seg_len, grads


def resnet18_like(M=8, step=0, config=2, device="cpu", pad_value=float("nan"), decay=0.7):
    """Config 2: per-tensor N(0, sigma_l^2), sigma_l log-uniform in [1e-5, 1e-2] (drawn once from
    seed 1000*config), every sigma scaled by decay^step so the norm falls faster than
    sqrt(alpha) and the bit rule walks down."""
    seg_len = resnet18_cifar10_segments()
    starts, _ = seg_starts(seg_len)
    rs = np.random.default_rng(1000 * config)
    sigma = 10.0 ** rs.uniform(-5.0, -2.0, size=len(seg_len))
    grads = _alloc(seg_len, M, device, pad_value)
    for i in range(M):
        gen = _gen(1000 * config + i + 100_000 * step, device)
        for l, (st, n) in enumerate(zip(starts, seg_len)):
            grads[i, st:st + n] = _normal(n, gen, device) * float(sigma[l] * decay ** step)
    return seg_len, grads


def transformer_like(M=16, config=3, device="cpu", pad_value=float("nan"), scale=1e-3, zero_rows=0.9):
    """Config 3: Laplace(0, scale) entries; the token embedding has `zero_rows` of its rows exactly
    zero, a fresh row subset per worker (tokens absent from the worker's batch)."""
    seg_len = transformer_classifier_segments()
    starts, _ = seg_starts(seg_len)
    grads = _alloc(seg_len, M, device, pad_value)
    for i in range(M):
        gen = _gen(1000 * config + i, device)
        for l, (st, n) in enumerate(zip(starts, seg_len)):
            x = _laplace(n, gen, device) * scale
            if l == 0:
                keep = torch.rand(30000, generator=gen, device=device) >= zero_rows
                x = (x.view(30000, 256) * keep[:, None].to(torch.float32)).reshape(-1)
            grads[i, st:st + n] = x
    return seg_len, grads


def flat_student_t(D=1 << 28, M=16, scale=1e-3, config=5, device="cpu", pad_value=float("nan"),
                   chunk=1 << 24):
    """Config 5: one tensor, heavy-tailed Student-t(nu=3) values times `scale`."""
    seg_len = [D]
    grads = _alloc(seg_len, M, device, pad_value)
    for i in range(M):
        gen = _gen(1000 * config + i, device)
        for c0 in range(0, D, chunk):
            n = min(chunk, D - c0)
            grads[i, c0:c0 + n] = _student_t3(n, gen, device).mul_(scale)
    return seg_len, grads


def ragged_mix(M=3, config=9, device="cpu", pad_value=float("nan")):
    """A small layout that exercises every edge of the padded index space: empty tensors, lengths
    around the 128 granule, a tensor spanning several tiles with a ragged tail."""
    seg_len = [1, 0, 127, 128, 129, 0, 0, 5, 2048, 4097, 3, 20000 + 77, 8192, 64]
    starts, _ = seg_starts(seg_len)
    grads = _alloc(seg_len, M, device, pad_value)
    for i in range(M):
        gen = _gen(1000 * config + i, device)
        for l, (st, n) in enumerate(zip(starts, seg_len)):
            if n:
                grads[i, st:st + n] = _student_t3(n, gen, device) * (10.0 ** (-(l % 5) - 1))
    return seg_len, grads


def logistic_regression_problem(n=262144, d=4096, config=4, device="cpu"):
    """Config 4: X ~ N(0,1), w* ~ N(0, I/d), y ~ Bernoulli(sigmoid(x.w*))."""
    gen = _gen(1000 * config, device)
    X = _normal(n * d, gen, device).view(n, d)
    w_star = _normal(d, gen, device) / math.sqrt(d)
    y = (torch.rand(n, generator=gen, device=device) < torch.sigmoid(X @ w_star)).to(torch.float32)
    return X, y, w_star
