"""Algorithm 1 of the paper (DQ-SGD in distributed learning) as a thin loop around the library.

Every numerical step of the hot path runs in the HIP kernels / C host code behind ``include/dq.h``:
``dq_norm`` (worker norms), ``dq_select_bits`` (Eq. (17)), ``dq_quantize_pack`` (Eq. (5)-(6)),
``dq_unpack_dequant_reduce_update`` (server average and x <- x - eta*g_hat), ``dq_alpha_est``
(Eq. (24)), ``dq_comm_cost_bits`` (Eq. (7)).  This module only sequences them the way Algorithm 1
does; the caller supplies the gradients (the training task is not part of this library).

Protocol (Algorithm 1 with the choices the paper leaves open):
  * lagged=True (the paper's): b_0 is an input; after iteration t the server computes b_{t+1}
    from iteration t's norms with index t+1, and only when (t+1) % tau == 0 (the paper updates the
    bit-width every tau iterations, tau = 100 in its experiments); otherwise b_{t+1} = b_t.
  * lagged=False: b_t is computed from iteration t's own norms before quantizing (needs the norms
    on the host before the quantize pass).
  * alpha: a number, or "estimate" to use Eq. (24) with the caller's loss at the update points.
  * per_tensor=True: one bit-width per tensor from ``dq_select_bits_per_tensor`` (b0, b_t in the
    result and on_step's b are then arrays of n_seg widths), messages in the per-tensor layout,
    through the ``*_v`` entry points.
  * With the lagged rule b_t is known before the gradient is looked at, so on a chunk-local plan
    (``plan.chunk_local``: no tensor crosses a multiple of 4096 padded elements, e.g. a gradient
    cut into buckets) the worker side is the single pass ``dq_norm_quantize_pack``; one_pass=False
    keeps the two calls.
  * norm_margin=m (base mode): from the second iteration on the worker side is the single
    pass ``dq_norm_quantize_pack_bracketed`` on any layout, every norm bracketed by the previous
    iteration's norm times (1 -+ m); the messages are the same as with the two calls whatever m
    is, a bracket that misses only costs time.  With lagged=False the pass is taken when both ends
    of the bracket give the same b_t (Eq. (17) is monotone in the norms); b_t is checked against
    the true norms afterwards and the quantization repeated if it moved.
  * per_worker=True: every worker takes Eq. (17) with its own norm (``dq_select_bits_per_worker``;
    with per_tensor=True also one width per tensor); b_t in the result are [M][n_seg] arrays.
  * device_rule=True: the rule runs on the GPU (``dq_select_bits_device``) and the loop never waits
    for the host; b_t and the cost are read back once at the end.  alpha must be a number.  With the
    lagged rule and norm_margin the worker side is ``dq_norm_quantize_pack_bracketed_v``: one pass
    over the gradient with the widths table the rule left on the GPU.
  * p: 2 or "inf", the norm of Eq. (5) (the paper leaves p open): ``dq_norm``/``dq_select_bits`` or
    ``dq_norm_linf``/``dq_select_bits_linf``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Union

import numpy as _np
import torch

from . import binding as _b


# Table 1 of the paper ("Parameters"): iterations, learning rate, batch size, and the two DQ-SGD
# hyper-parameters k and alpha per task; W = 8 workers and tau = 100 throughout (Section 6).  The
# paper never defines k; the only free constant of Eq. (17) besides alpha is sqrt(T / eps_hat_Q),
# so k is read as that factor: s*_t = k * alpha^((T-1-t)/2) * G-bar_t, eps_hat_Q = T / k^2.
PAPER_PRESETS = {
    "ag_news_bilstm": dict(T=1000, eta=0.005, batch=32, k=5.0, alpha=0.994, W=8, tau=100),
    "cifar10_resnet18": dict(T=6000, eta=0.1, batch=32, k=20.0, alpha=0.999, W=8, tau=100),
    "cifar100_resnet34": dict(T=6000, eta=0.01, batch=64, k=10.0, alpha=0.999, W=8, tau=100),
}


def eps_hat_from_k(T: int, k: float) -> float:
    """eps_hat_Q for which sqrt(T / eps_hat_Q) = k (the reading of Table 1's k stated above)."""
    if T < 1 or not k > 0:
        raise ValueError("T >= 1 and k > 0")
    return T / (k * k)


@dataclass
class DQSGDResult:
    x: "torch.Tensor"                      # x_T, padded layout
    bits: List[int] = field(default_factory=list)       # b_t used at every iteration
    gbar: List[float] = field(default_factory=list)     # G-bar_t
    cost_bits: int = 0                                   # f_Q of Eq. (7), summed over iterations
    alphas: List[float] = field(default_factory=list)   # alpha used at each bit update


def run(plan: _b.Plan, x0: "torch.Tensor", grad_fn: Callable[[int, "torch.Tensor", "torch.Tensor"], None],
        M: int, T: int, eta: float, eps_hat_q: float, alpha: Union[float, str], b0: int,
        b_min: int = 1, b_max: int = 8, tau: int = 1, lagged: bool = True, seed: int = 0,
        loss_fn: Optional[Callable[["torch.Tensor"], float]] = None, B_pre: int = 32,
        on_step: Optional[Callable] = None, p: Union[int, str] = 2, per_tensor: bool = False,
        device_rule: bool = False, one_pass: bool = True, per_worker: bool = False,
        norm_margin: Optional[float] = None) -> DQSGDResult:
    """grad_fn(t, x, grads_out) fills grads_out[M][D'] (float32, CUDA, padded layout) with the M
    workers' stochastic gradients at x.  on_step(t, b_t, grads, norms_host, packed) is called after
    the quantize pass of every iteration (tests use it to feed the same bytes to the oracle)."""
    if p not in (2, "inf"):
        raise ValueError('p must be 2 or "inf"')
    norm_fn, rule = (_b.norm, _b.select_bits) if p == 2 else (_b.norm_linf, _b.select_bits_linf)
    dp, n_seg = plan.padded_elems, plan.n_seg
    if per_worker:
        if device_rule or p != 2:
            raise ValueError("per_worker runs the host rule with the l2 norm")
        return _run_per_worker(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged,
                               seed, B_pre, on_step, per_tensor, one_pass and lagged and plan.chunk_local)
    if device_rule:
        if per_tensor and p != 2:
            raise ValueError("per_tensor uses the tensors' own norms: leave p at 2 or run the max norm without it")
        rule_name = "per_tensor" if per_tensor else ("single" if p == 2 else "single_linf")
        return _run_device_rule(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged,
                                seed, B_pre, on_step, norm_fn, rule_name, norm_margin)
    if per_tensor:
        return _run_per_tensor(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged,
                               seed, B_pre, on_step, norm_fn, one_pass and lagged and plan.chunk_local, p != 2)
    dev = x0.device
    x = x0.clone()
    grads = torch.zeros((M, dp), dtype=torch.float32, device=dev)
    norms = torch.empty((M, n_seg), dtype=torch.float32, device=dev)
    norms_host = torch.empty((M, n_seg), dtype=torch.float32).pin_memory()
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device=dev)
    packed = torch.zeros((M, plan.packed_bytes(b_max)), dtype=torch.uint8, device=dev)
    d_true = int(plan.seg_len.sum())
    res = DQSGDResult(x=x)
    estimate = alpha == "estimate"
    if estimate and (loss_fn is None or not lagged):
        raise ValueError('alpha="estimate" needs loss_fn and the lagged protocol')
    F0 = loss_fn(x) if estimate else None
    cur_alpha = 1.0 if estimate else float(alpha)
    b = int(b0)

    single_pass = one_pass and lagged and plan.chunk_local
    bracketed = norm_margin is not None and not single_pass
    if bracketed:
        if not 0.0 <= norm_margin < 1.0:
            raise ValueError("norm_margin must be in [0, 1)")
        wsb = torch.empty(_b.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device=dev)
        prev, lo, hi = (torch.empty_like(norms) for _ in range(3))
    for t in range(T):
        grad_fn(t, x, grads)
        pk = None
        if single_pass:
            pk = packed[:, :plan.packed_bytes(b)]
            _b.norm_quantize_pack(plan, grads, b, seed, t, norms, pk, linf=p != 2)
        elif bracketed and t > 0:
            _b.norm_bracket(prev, norm_margin, lo, hi)
            b_guess = b
            if not lagged:
                # Eq. (17) never decreases in any norm, so if both ends of the bracket give the same b,
                # every set of norms inside it does; the ends are the ones dq_norm_bracket has just written.
                b_lo = rule(lo.cpu().numpy(), t, T, eps_hat_q, cur_alpha, b_min, b_max)[0]
                b_hi = rule(hi.cpu().numpy(), t, T, eps_hat_q, cur_alpha, b_min, b_max)[0]
                b_guess = b_lo if b_lo == b_hi else None
            if b_guess is None:
                norm_fn(plan, grads, norms, ws)
            else:
                pk = packed[:, :plan.packed_bytes(b_guess)]
                _b.norm_quantize_pack_bracketed(plan, grads, lo, hi, b_guess, seed, t, norms, pk, wsb, linf=p != 2)
        else:
            norm_fn(plan, grads, norms, ws)
        if bracketed:
            prev.copy_(norms)
        norms_host.copy_(norms, non_blocking=True)
        if not lagged:
            torch.cuda.current_stream().synchronize()
            b, gb = rule(norms_host.numpy(), t, T, eps_hat_q, cur_alpha, b_min, b_max)
            if pk is not None and b != b_guess:   # a norm left its bracket and moved b: quantize again
                pk = None
        if pk is None:
            pk = packed[:, :plan.packed_bytes(b)]
            _b.quantize_pack(plan, grads, norms, b, seed, t, pk)
        if on_step is not None:
            torch.cuda.current_stream().synchronize()
            on_step(t, b, grads, norms_host.numpy(), pk)
        _b.unpack_dequant_reduce_update(plan, pk, norms, b, eta, x)
        res.bits.append(b)
        res.cost_bits += _b.comm_cost_bits(M, d_true, b, n_seg, B_pre)
        if lagged:
            torch.cuda.current_stream().synchronize()
            gb = rule(norms_host.numpy(), t, T, eps_hat_q, 1.0, b_min, b_max)[1]
            if t + 1 < T and (t + 1) % tau == 0:
                if estimate:
                    cur_alpha = min(1.0, _b.alpha_est(loss_fn(x), F0, t + 1))
                    res.alphas.append(cur_alpha)
                b, _ = rule(norms_host.numpy(), t + 1, T, eps_hat_q, cur_alpha, b_min, b_max)
        res.gbar.append(gb)
    torch.cuda.synchronize()
    return res


def _run_per_tensor(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged, seed, B_pre,
                    on_step, norm_fn, single_pass=False, linf=False) -> DQSGDResult:
    import numpy as np
    if alpha == "estimate":
        raise ValueError('alpha="estimate" is not available with per_tensor')
    dp, n_seg = plan.padded_elems, plan.n_seg
    dev = x0.device
    x = x0.clone()
    grads = torch.zeros((M, dp), dtype=torch.float32, device=dev)
    norms = torch.empty((M, n_seg), dtype=torch.float32, device=dev)
    norms_host = torch.empty((M, n_seg), dtype=torch.float32).pin_memory()
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device=dev)
    packed = torch.zeros((M, _b.packed_bytes_v(plan, [b_max] * n_seg)), dtype=torch.uint8, device=dev)
    b = np.broadcast_to(np.asarray(b0, dtype=np.int32), (n_seg,)).copy()
    table = _b.Widths(plan, b)
    res = DQSGDResult(x=x)
    for t in range(T):
        grad_fn(t, x, grads)
        if single_pass:
            pk = packed[:, :table.packed_bytes]
            _b.norm_quantize_pack_v(plan, table, grads, seed, t, norms, pk, linf=linf)
        else:
            norm_fn(plan, grads, norms, ws)
        norms_host.copy_(norms, non_blocking=True)
        if not lagged:
            torch.cuda.current_stream().synchronize()
            b, _ = _b.select_bits_per_tensor(norms_host.numpy(), t, T, eps_hat_q, float(alpha), b_min, b_max)
            table.set(b)
        if not single_pass:
            pk = packed[:, :table.packed_bytes]
            _b.quantize_pack_v(plan, table, grads, norms, seed, t, pk)
        if on_step is not None:
            torch.cuda.current_stream().synchronize()
            on_step(t, b.copy(), grads, norms_host.numpy(), pk)
        _b.unpack_dequant_reduce_update_v(plan, table, pk, norms, eta, x)
        res.bits.append(b.copy())
        res.cost_bits += _b.comm_cost_bits_per_tensor(M, plan.seg_len, b, B_pre)
        torch.cuda.current_stream().synchronize()
        res.gbar.append(_b.select_bits(norms_host.numpy(), t, T, eps_hat_q, float(alpha), b_min, b_max)[1])  # G-bar_t of Lemma 1
        if lagged and t + 1 < T and (t + 1) % tau == 0:
            b, _ = _b.select_bits_per_tensor(norms_host.numpy(), t + 1, T, eps_hat_q, float(alpha), b_min, b_max)
            table.set(b)
    torch.cuda.synchronize()
    table.close()
    return res


def _run_device_rule(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged, seed, B_pre,
                     on_step, norm_fn, rule_name, norm_margin=None) -> DQSGDResult:
    import numpy as np
    if alpha == "estimate":
        raise ValueError('alpha="estimate" needs the loss on the host: not available with device_rule')
    alpha = float(alpha)
    dp, n_seg = plan.padded_elems, plan.n_seg
    dev = x0.device
    x = x0.clone()
    grads = torch.zeros((M, dp), dtype=torch.float32, device=dev)
    norms = torch.empty((M, n_seg), dtype=torch.float32, device=dev)
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device=dev)
    packed = torch.zeros((M, _b.packed_bytes_v(plan, [b_max] * n_seg)), dtype=torch.uint8, device=dev)
    # per iteration: the widths used and G-bar (single rules) / the tensors' Nbar (per tensor)
    b_hist = torch.zeros((T, n_seg), dtype=torch.int32, device=dev)
    g_cols = n_seg if rule_name == "per_tensor" else 1
    g_hist = torch.zeros((T, g_cols), dtype=torch.float64, device=dev)
    b_cur = torch.from_numpy(np.broadcast_to(np.asarray(b0, dtype=np.int32), (n_seg,)).copy()).to(dev)
    table = _b.Widths(plan, b_cur.cpu().numpy())
    unused = _b.Widths(plan)
    # With the lagged rule the widths are on the GPU before the gradient exists; with a margin for
    # the norms as well, norms and messages come from one pass and nothing in the loop waits for the host.
    bracketed = norm_margin is not None and lagged
    if bracketed:
        if not 0.0 <= norm_margin < 1.0:
            raise ValueError("norm_margin must be in [0, 1)")
        wsb = torch.empty(_b.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device=dev)
        prev, lo, hi = (torch.empty_like(norms) for _ in range(3))
    for t in range(T):
        grad_fn(t, x, grads)
        one_pass = bracketed and t > 0
        if one_pass:
            _b.norm_bracket(prev, norm_margin, lo, hi)
            _b.norm_quantize_pack_bracketed_v(plan, table, grads, lo, hi, seed, t, norms, packed, wsb,
                                              linf=rule_name == "single_linf")
        else:
            norm_fn(plan, grads, norms, ws)
        if bracketed:
            prev.copy_(norms)
        if not lagged:
            _b.select_bits_device(plan, table, norms, t, T, eps_hat_q, alpha, b_min, b_max, rule=rule_name,
                                  b_out=b_hist[t], gbar_out=g_hist[t])
        else:
            b_hist[t].copy_(b_cur)
        if not one_pass:
            _b.quantize_pack_v(plan, table, grads, norms, seed, t, packed)
        if on_step is not None:
            torch.cuda.current_stream().synchronize()
            b_now = b_hist[t].cpu().numpy()
            on_step(t, b_now if rule_name == "per_tensor" else int(b_now[0]), grads, norms.cpu().numpy(),
                    packed[:, :_b.packed_bytes_v(plan, b_now)])
        _b.unpack_dequant_reduce_update_v(plan, table, packed, norms, eta, x)
        if lagged:
            # at the update points b_{t+1} comes from these norms with index t+1; otherwise the rule
            # only serves the record of G-bar and fills a table nothing reads
            if t + 1 < T and (t + 1) % tau == 0:
                _b.select_bits_device(plan, table, norms, t + 1, T, eps_hat_q, alpha, b_min, b_max,
                                      rule=rule_name, b_out=b_cur, gbar_out=g_hist[t])
            else:
                _b.select_bits_device(plan, unused, norms, t, T, eps_hat_q, alpha, b_min, b_max,
                                      rule=rule_name, gbar_out=g_hist[t])
    torch.cuda.synchronize()
    table.close()
    unused.close()
    res = DQSGDResult(x=x)
    b_host = b_hist.cpu().numpy()
    g_host = g_hist.cpu().numpy()
    for t in range(T):
        if rule_name == "per_tensor":
            res.bits.append(b_host[t].copy())
            res.cost_bits += _b.comm_cost_bits_per_tensor(M, plan.seg_len, b_host[t], B_pre)
            res.gbar.append(float(np.sqrt((g_host[t] ** 2).sum())))
        else:
            res.bits.append(int(b_host[t, 0]))
            res.cost_bits += _b.comm_cost_bits(M, int(plan.seg_len.sum()), int(b_host[t, 0]), n_seg, B_pre)
            res.gbar.append(float(g_host[t, 0]))
    return res


def _run_per_worker(plan, x0, grad_fn, M, T, eta, eps_hat_q, alpha, b0, b_min, b_max, tau, lagged, seed, B_pre,
                    on_step, per_tensor, single_pass) -> DQSGDResult:
    import numpy as np
    if alpha == "estimate":
        raise ValueError('alpha="estimate" is not available with per_worker')
    dp, n_seg = plan.padded_elems, plan.n_seg
    dev = x0.device
    x = x0.clone()
    grads = torch.zeros((M, dp), dtype=torch.float32, device=dev)
    norms = torch.empty((M, n_seg), dtype=torch.float32, device=dev)
    norms_host = torch.empty((M, n_seg), dtype=torch.float32).pin_memory()
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device=dev)
    packed = torch.zeros((M, _b.packed_bytes_v(plan, [b_max] * n_seg)), dtype=torch.uint8, device=dev)
    b = np.broadcast_to(np.asarray(b0, dtype=np.int32), (M, n_seg)).copy()
    table = _b.Widths(plan, b, workers=M)
    res = DQSGDResult(x=x)
    for t in range(T):
        grad_fn(t, x, grads)
        if single_pass:
            _b.norm_quantize_pack_v(plan, table, grads, seed, t, norms, packed)
        else:
            _b.norm(plan, grads, norms, ws)
        norms_host.copy_(norms, non_blocking=True)
        if not lagged:
            torch.cuda.current_stream().synchronize()
            b = _b.select_bits_per_worker(norms_host.numpy(), t, T, eps_hat_q, float(alpha), b_min, b_max, per_tensor)
            table.set(b)
        if not single_pass:
            _b.quantize_pack_v(plan, table, grads, norms, seed, t, packed)
        if on_step is not None:
            torch.cuda.current_stream().synchronize()
            on_step(t, b.copy(), grads, norms_host.numpy(), packed[:, :table.packed_bytes])
        _b.unpack_dequant_reduce_update_v(plan, table, packed, norms, eta, x)
        res.bits.append(b.copy())
        res.cost_bits += sum(_b.comm_cost_bits_per_tensor(1, plan.seg_len, b[i], B_pre) for i in range(M))
        torch.cuda.current_stream().synchronize()
        res.gbar.append(_b.select_bits(norms_host.numpy(), t, T, eps_hat_q, float(alpha), b_min, b_max)[1])  # G-bar_t of Lemma 1
        if lagged and t + 1 < T and (t + 1) % tau == 0:
            b = _b.select_bits_per_worker(norms_host.numpy(), t + 1, T, eps_hat_q, float(alpha), b_min, b_max,
                                          per_tensor)
            table.set(b)
    torch.cuda.synchronize()
    table.close()
    return res
