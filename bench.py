#!/usr/bin/env python3
"""Benchmark of the DQ-SGD quantizer hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic gradients that are already
resident in HBM:  dq_norm -> (norms to host) -> dq_select_bits -> dq_quantize_pack (all M workers)
-> dq_unpack_dequant_reduce.  The default workload is the large flat gradient of the headline metric
(D = 2^28 fp32 per worker, M = 16, Student-t(3) * 1e-3, b_t from the dynamic rule in 2..8), the
one the >= 70 %-of-HBM target is quoted on.

Prints ONE JSON line: whole-step throughput in GB/s of fp32 input, the roofline of the dominant
kernel (quantize+pack) from HIP-event timings taken inside the timed region, per-kernel figures,
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published


def make_workload(name: str, M: int | None, log2d: int | None):
    from paper_2107_14575_amd import workloads as wl
    if name == "flat_student_t":
        D = 1 << (log2d or 28)
        seg_len, grads = wl.flat_student_t(D=D, M=M or 16, device="cuda")
        label = f"flat fp32 gradient D=2^{log2d or 28}, Student-t(nu=3)*1e-3, M={M or 16}, b_t dynamic in 2..8"
    elif name == "resnet18":
        seg_len, grads = wl.resnet18_like(M=M or 8, device="cuda")
        label = f"ResNet-18-shaped gradient, 62 tensors, 11.17M params, M={M or 8}, b_t dynamic in 2..8"
    elif name == "transformer":
        seg_len, grads = wl.transformer_like(M=M or 16, device="cuda")
        label = f"Transformer-classifier-shaped gradient, 102 tensors, 12.55M params, M={M or 16}, b_t dynamic in 2..8"
    elif name == "flat_gaussian":
        D = 1 << (log2d or 20)
        seg_len, grads = wl.flat_gaussian(D=D, M=M or 4, device="cuda")
        label = f"flat fp32 gradient D=2^{log2d or 20}, N(0,1e-6), M={M or 4}, b_t dynamic in 2..8"
    else:
        raise SystemExit(f"unknown workload {name}")
    return seg_len, grads, label


def cpu_baseline(seg_len, grads_dev, b: int, target_elems: int, n_steps: int):
    """The oracle as it stands, timed on the host over a bounded sample: the first
    min(D', target) elements of every worker of the same workload (single-tensor workloads) or the
    whole gradient when it is small.  n_steps full steps (norm + quantize+pack +
    unpack+dequant+average, the step index advancing as in Algorithm 1), about 10 s of host work
    at the defaults."""
    import numpy as np
    from oracle import dqo
    from paper_2107_14575_amd import workloads as wl

    M = grads_dev.shape[0]
    _, dp = wl.seg_starts(seg_len)
    if len(seg_len) == 1 and seg_len[0] > target_elems:
        n = target_elems
        sample_seg = [n]
        g = np.ascontiguousarray(grads_dev[:, :n].cpu().numpy())
        what = f"first 2^{n.bit_length() - 1} elements of each of the {M} workers"
    else:
        sample_seg = list(seg_len)
        g = np.ascontiguousarray(grads_dev.cpu().numpy())
        what = f"the whole gradient of each of the {M} workers"
    dqo.build()
    threads = dqo.num_threads()
    t0 = time.perf_counter()
    for step in range(n_steps):
        norms = dqo.norm(sample_seg, g)
        packed = dqo.quantize_pack(sample_seg, g, norms, b, wl.QUANT_SEED, step)
        out = dqo.unpack_dequant_reduce(sample_seg, packed, norms, b)
    dt = time.perf_counter() - t0
    assert out.shape[0] == wl.seg_starts(sample_seg)[1]
    n_in = n_steps * M * sum(sample_seg) * 4
    return {"value": round(n_in / dt / 1e9, 4), "unit": "GB/s of fp32 input", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"{n_steps} steps (norm, quantize+pack, unpack+dequant+average) at b={b} on {what}"}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="flat_student_t",
                    choices=["flat_student_t", "resnet18", "transformer", "flat_gaussian"])
    ap.add_argument("--workers", type=int, default=None)
    ap.add_argument("--log2d", type=int, default=None)
    ap.add_argument("--fixed-bits", type=int, default=0, help="use this b every step instead of the rule")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=26)
    ap.add_argument("--cpu-steps", type=int, default=5, help="steps of the oracle timed for cpu_baseline")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region, one plain device copy of the output buffer (4*D' bytes "
                         "read, 4*D' written): the known-size reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build measures the one-GPU hot path only (M workers simulated in-device); "
                         "run with --gpus 1")

    import numpy as np
    import torch

    import paper_2107_14575_amd as dq
    from paper_2107_14575_amd import workloads as wl

    dq.load_library()
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    torch.cuda.set_device(0)

    seg_len, grads, label = make_workload(args.workload, args.workers, args.log2d)
    if args.fixed_bits:
        label = label.replace("b_t dynamic in 2..8", f"b = {args.fixed_bits} fixed")
    M, stride = grads.shape
    D = sum(seg_len)
    plan = dq.Plan(seg_len)
    dp = plan.padded_elems
    n_seg = plan.n_seg
    norms_dev = torch.empty((M, n_seg), dtype=torch.float32, device="cuda")
    norms_host = torch.empty((M, n_seg), dtype=torch.float32).pin_memory()
    ws = torch.empty(plan.workspace_bytes(M), dtype=torch.uint8, device="cuda")
    packed = torch.zeros((M, plan.packed_bytes(8)), dtype=torch.uint8, device="cuda")
    out = torch.empty(dp, dtype=torch.float32, device="cuda")

    # constants of the bit rule: alpha = 0.9, T = warmup + steps, eps_hat such that the rule sits
    # at s* = 0.9 * 15 (b = 4) at the last step for this workload's Gbar
    T = args.warmup + args.steps
    alpha = 0.9
    dq.norm(plan, grads, norms_dev, ws)
    torch.cuda.synchronize()
    n0 = norms_dev.cpu().numpy().astype(np.float64)
    gbar0 = float(np.sqrt((n0 ** 2).sum() / M))
    eps_hat = T * (gbar0 / (0.9 * 15.0)) ** 2 if gbar0 > 0 else 1.0

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []  # per timed step: (b, [e0, e1, e2, e3, e4])

    def step(t: int, timed: bool):
        e = [ev() for _ in range(5)] if timed else None
        if timed: e[0].record()
        dq.norm(plan, grads, norms_dev, ws)
        if timed: e[1].record()
        norms_host.copy_(norms_dev, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        if args.fixed_bits:
            b = args.fixed_bits
        else:
            b, _ = dq.select_bits(norms_host.numpy(), t, T, eps_hat, alpha, 2, 8)
        pk = packed[:, :plan.packed_bytes(b)]
        if timed: e[2].record()
        dq.quantize_pack(plan, grads, norms_dev, b, wl.QUANT_SEED, t, pk)
        if timed: e[3].record()
        dq.unpack_dequant_reduce(plan, pk, norms_dev, b, out)
        if timed:
            e[4].record()
            marks.append((b, e))
        return b

    for t in range(args.warmup):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup, T):
        step(t, True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    def timed_loop(fn, reps: int = 5, warm: int = 1) -> float:
        """ms per call, after `warm` untimed calls, with events on the stream the kernels run on"""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        u0, u1 = ev(), ev()
        u0.record()
        for _ in range(reps):
            fn()
        u1.record()
        torch.cuda.synchronize()
        return u0.elapsed_time(u1) / reps

    # the other entry points on the same data, each timed on its own (not part of `value`)
    b_last = marks[-1][0]
    pk_last = packed[:, :plan.packed_bytes(b_last)]
    # reduce fused with the model update of Algorithm 1 (x <- x - eta*g_hat)
    x_model = torch.zeros(dp, dtype=torch.float32, device="cuda")
    t_upd = timed_loop(lambda: dq.unpack_dequant_reduce_update(plan, pk_last, norms_dev, b_last, 1e-3, x_model))
    del x_model
    # max-norm variant of the norm pass (p = infinity in Eq. (5))
    norms_inf = torch.empty_like(norms_dev)
    t_ninf = timed_loop(lambda: dq.norm_linf(plan, grads, norms_inf, ws))
    # per-tensor-width kernels at the same widths (every tensor b_last)
    table = dq.Widths(plan, [b_last] * n_seg)
    t_qv = timed_loop(lambda: dq.quantize_pack_v(plan, table, grads, norms_dev, wl.QUANT_SEED, T, pk_last))
    t_rv = timed_loop(lambda: dq.unpack_dequant_reduce_v(plan, table, pk_last, norms_dev, out))
    table.close()
    # the reduce with a widths table that has one row per worker (here all rows equal)
    table_w = dq.Widths(plan, [[b_last] * n_seg] * M, workers=M)
    t_rw = timed_loop(lambda: dq.unpack_dequant_reduce_v(plan, table_w, pk_last, norms_dev, out))
    table_w.close()
    # sign-only baseline (one bit per element)
    sign_msgs = packed[:, :dp // 8]
    t_sp = timed_loop(lambda: dq.sign_pack(plan, grads, sign_msgs))
    t_sr = timed_loop(lambda: dq.sign_reduce(plan, sign_msgs, out))
    t_sm = timed_loop(lambda: dq.sign_majority(plan, sign_msgs, out))
    t_ss = timed_loop(lambda: dq.sign_reduce(plan, sign_msgs, out, scales=norms_dev))
    # the whole step with the rule evaluated on the GPU (no host round trip; per-tensor-width kernels)
    table = dq.Widths(plan)
    b_dev = torch.zeros(n_seg, dtype=torch.int32, device="cuda")

    def device_rule_step(t):
        dq.norm(plan, grads, norms_dev, ws)
        dq.select_bits_device(plan, table, norms_dev, t, T, eps_hat, alpha, 2, 8, rule="single", b_out=b_dev)
        dq.quantize_pack_v(plan, table, grads, norms_dev, wl.QUANT_SEED, t, packed)
        dq.unpack_dequant_reduce_v(plan, table, packed, norms_dev, out)

    device_rule_step(T - 1)
    torch.cuda.synchronize()
    t0_dev = time.perf_counter()
    for t in range(args.warmup, T):
        device_rule_step(t)
    torch.cuda.synchronize()
    ms_device_rule = (time.perf_counter() - t0_dev) / args.steps * 1e3
    assert int(b_dev[0]) == b_last, "device rule and host rule disagree"
    table.close()
    # The paper's own protocol between bit updates (b_t received from the server beforehand), on the
    # same gradient cut into 4096-element buckets with one norm each: norms and messages in ONE
    # pass over the gradient (dq_norm_quantize_pack), then the reduce.
    one_pass = None
    if n_seg == 1 and D % 4096 == 0:
        bplan = dq.Plan([4096] * (D // 4096))
        bnorms = torch.empty((M, bplan.n_seg), dtype=torch.float32, device="cuda")
        t_fused = timed_loop(lambda: dq.norm_quantize_pack(bplan, grads, b_last, wl.QUANT_SEED, T, bnorms, pk_last))
        t_bred = timed_loop(lambda: dq.unpack_dequant_reduce(bplan, pk_last, bnorms, b_last, out))

        def lagged_step(t):
            dq.norm_quantize_pack(bplan, grads, b_last, wl.QUANT_SEED, t, bnorms, pk_last)
            dq.unpack_dequant_reduce(bplan, pk_last, bnorms, b_last, out)

        lagged_step(0)
        torch.cuda.synchronize()
        t0_l = time.perf_counter()
        for t in range(args.steps):
            lagged_step(t)
        torch.cuda.synchronize()
        ms_lagged = (time.perf_counter() - t0_l) / args.steps * 1e3
        one_pass = (t_fused, t_bred, ms_lagged, bplan.n_seg)
        bplan.close()
        del bnorms
    # The same protocol on the benchmark's own layout (one norm for the whole gradient): norms and
    # messages in ONE pass given a bracket for every norm -- here the norms of the step before, give or
    # take 12.5 % -- then the reduce.  Elements the bracket leaves open are settled afterwards.
    wsb = torch.empty(dq.bracketed_workspace_bytes(plan, M), dtype=torch.uint8, device="cuda")
    br_stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    br_norms = torch.empty_like(norms_dev)
    br_lo, br_hi = torch.empty_like(norms_dev), torch.empty_like(norms_dev)
    dq.norm_bracket(norms_dev, 0.125, br_lo, br_hi)
    t_br = timed_loop(lambda: dq.norm_quantize_pack_bracketed(plan, grads, br_lo, br_hi, b_last, wl.QUANT_SEED, T,
                                                              br_norms, pk_last, wsb, stats=br_stats))

    def bracketed_step(t):
        dq.norm_quantize_pack_bracketed(plan, grads, br_lo, br_hi, b_last, wl.QUANT_SEED, t, br_norms, pk_last, wsb)
        dq.unpack_dequant_reduce(plan, pk_last, br_norms, b_last, out)

    bracketed_step(0)
    torch.cuda.synchronize()
    t0_b = time.perf_counter()
    for t in range(args.steps):
        bracketed_step(t)
    torch.cuda.synchronize()
    ms_bracketed = (time.perf_counter() - t0_b) / args.steps * 1e3
    br_counts = [int(v) for v in br_stats.tolist()]
    # Algorithm 1's protocol end to end on the GPU: the widths table was filled by the rule at the end of the
    # iteration before (lagged b), this iteration reads the gradients once, the server reduces, then the
    # rule decides the next iteration's width -- no host round trip anywhere in the step.
    table = dq.Widths(plan, [b_last] * n_seg)
    b_dev2 = torch.zeros(n_seg, dtype=torch.int32, device="cuda")

    def lagged_device_step(t):
        dq.norm_quantize_pack_bracketed_v(plan, table, grads, br_lo, br_hi, wl.QUANT_SEED, t, br_norms, packed, wsb)
        dq.unpack_dequant_reduce_v(plan, table, packed, br_norms, out)
        dq.select_bits_device(plan, table, br_norms, min(t + 1, T - 1), T, eps_hat, alpha, 2, 8, rule="single",
                              b_out=b_dev2)

    lagged_device_step(T - 1)
    torch.cuda.synchronize()
    t0_ld = time.perf_counter()
    for t in range(args.warmup, T):
        lagged_device_step(t)
    torch.cuda.synchronize()
    ms_lagged_device = (time.perf_counter() - t0_ld) / args.steps * 1e3
    table.close()
    del wsb
    # leave packed/out as the last step left them for anything that follows
    dq.quantize_pack(plan, grads, norms_dev, b_last, wl.QUANT_SEED, T - 1, pk_last)
    dq.unpack_dequant_reduce(plan, pk_last, norms_dev, b_last, out)
    torch.cuda.synchronize()

    if args.copy_probe:
        probe = torch.empty_like(out)
        probe.copy_(out)
        torch.cuda.synchronize()

    def independent_ceiling(reps: int = 5):
        """GB/s (read + written) that kernels this repository did not write reach on the same buffers,
        one per read/write mix: torch's elementwise kernels and fill, and the HIP runtime's device copy.
        They read the gradients (up to 2^30 elements, far beyond the 256 MB last-level cache) and write
        into the message / output buffers, whose contents bench.py restores afterwards."""
        n = min(grads.numel(), 1 << 30)
        src = grads.reshape(-1)[:n]
        flat = packed.reshape(-1)
        if flat.numel() < 2 * n or n < (1 << 26):
            return None
        as_bool, as_half = flat[:n].view(torch.bool), flat[:2 * n].view(torch.float16)
        n_out = min(n, out.numel())
        cases = {
            "fp32 -> bool  (torch.lt, 4 B read : 1 B written)": (lambda: torch.lt(src, 0, out=as_bool), 4 * n, n),
            "fp32 -> fp16  (Tensor.copy_, 4 : 2)": (lambda: as_half.copy_(src), 4 * n, 2 * n),
            "fp32 -> fp32  (torch.neg, 4 : 4)": (lambda: torch.neg(src[:n_out], out=out[:n_out]), 4 * n_out, 4 * n_out),
            "fp16 -> fp32  (Tensor.copy_, 2 : 4)": (lambda: out[:n_out].copy_(as_half[:n_out]), 2 * n_out, 4 * n_out),
            "device copy   (Tensor.copy_ fp32, hipMemcpy, 4 : 4)": (lambda: out[:n_out].copy_(src[:n_out]), 4 * n_out, 4 * n_out),
            "fill          (Tensor.zero_, write only)": (lambda: as_half.zero_(), 0, 2 * n),
        }
        res = {}
        for name, (fn, rd, wr) in cases.items():
            ms = timed_loop(fn, reps)
            res[name] = {"GBps": round((rd + wr) / ms / 1e6, 1), "frac_of_peak": round((rd + wr) / ms / 1e6 / HBM_PEAK_GBS, 4),
                         "written_per_read": round(wr / rd, 4) if rd else None, "ms": round(ms, 4)}
        return res

    ms_per_step = elapsed / args.steps * 1e3
    in_bytes = M * D * 4
    value = in_bytes / (elapsed / args.steps) / 1e9

    bits = [b for b, _ in marks]
    t_norm = sum(e[0].elapsed_time(e[1]) for _, e in marks) / len(marks)
    t_quant = sum(e[2].elapsed_time(e[3]) for _, e in marks) / len(marks)
    t_red = sum(e[3].elapsed_time(e[4]) for _, e in marks) / len(marks)
    # algorithmic bytes per launch (padded elements are moved too; D' == D for the flat workloads)
    q_bytes = sum(M * dp * (4 + (b + 1) / 8) for b in bits) / len(bits)
    r_bytes = sum(dp * (M * (b + 1) / 8 + 4) for b in bits) / len(bits)
    n_bytes = M * dp * 4

    def rl(bytes_, ms):
        a = bytes_ / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(a / HBM_PEAK_GBS, 4), "traffic": None, "avg_ms": round(ms, 4),
                "algorithmic_bytes_per_launch": int(bytes_)}

    def profiled_traffic(kernel_tag: str):
        """HBM bytes per launch from the committed rocprofv3 counter summaries of this kernel on this
        workload (FETCH_SIZE and WRITE_SIZE passes of their own, each scaled by a plain device copy; the
        counters cannot be read from inside this process): the per-width table `..._b1to8.txt`, weighted
        by the widths of the timed steps; for kernels whose traffic does not depend on b the
        single-width summary.  None when no summary covers the workload."""
        import re
        shape = f"flat_student_t_d2p{dp.bit_length() - 1}_m{M}" if args.workload == "flat_student_t" else f"{args.workload}_m{M}"
        pdir = os.path.join(ROOT, "profiles")
        table = os.path.join(pdir, f"{kernel_tag}__{shape}_b1to8.txt")
        if os.path.exists(table):
            rows = {}
            for line in open(table):
                f = line.split()
                if len(f) >= 9 and f[0].isdigit() and f[1].isdigit():
                    rows[int(f[0])] = (float(f[6]), float(f[7]))  # HBM GB read, written
            if all(b in rows for b in bits):
                rd = sum(rows[b][0] for b in bits) / len(bits)
                wr = sum(rows[b][1] for b in bits) / len(bits)
                return {"bytes": int((rd + wr) * 1e9), "read_GB": round(rd, 4), "written_GB": round(wr, 4),
                        "source": "profiles/" + os.path.basename(table) + ", rows weighted by b_t"}
        for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
            if not re.fullmatch(re.escape(f"{kernel_tag}__{shape}_b") + r"\d\.txt", name):
                continue
            if kernel_tag not in ("k_norm_partial", "k_norm_partial_linf") and name != f"{kernel_tag}__{shape}_b{bits[0]}.txt":
                continue
            if kernel_tag not in ("k_norm_partial", "k_norm_partial_linf") and len(set(bits)) != 1:
                continue
            text = open(os.path.join(pdir, name)).read()
            rd = re.search(r"FETCH_SIZE mean \d+ -> ([0-9.]+) GB read", text)
            wr = re.search(r"WRITE_SIZE mean \d+ -> ([0-9.]+) GB written", text)
            if rd and wr:
                return {"bytes": int((float(rd.group(1)) + float(wr.group(1))) * 1e9), "read_GB": float(rd.group(1)),
                        "written_GB": float(wr.group(1)), "source": "profiles/" + name}
        return None

    result = {
        "metric": "quantize+pack and unpack+dequant+reduce GB/s (fp32 in) and % of HBM peak",
        "value": round(value, 2),
        "unit": "GB/s of fp32 input (whole step: norm + select_bits + quantize+pack + unpack+dequant+reduce)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": label, "D": D, "padded_D": dp, "M": M, "n_tensors": n_seg,
                   "b_t": bits, "T": T, "alpha": alpha, "eps_hat_q": eps_hat, "Gbar": gbar0,
                   "seed": wl.QUANT_SEED},
        "roofline": dict(rl(q_bytes, t_quant), kernel="k_quantize_pack"),
        "kernels": {
            "dq_quantize_pack": dict(rl(q_bytes, t_quant), fp32_in_GBps=round(in_bytes / t_quant / 1e6, 1)),
            "dq_unpack_dequant_reduce": dict(rl(r_bytes, t_red), fp32_in_GBps=round(in_bytes / t_red / 1e6, 1)),
            "dq_norm": rl(n_bytes, t_norm),
            "dq_unpack_dequant_reduce_update": rl(dp * (M * (b_last + 1) / 8 + 8), t_upd),
            "dq_norm_linf": rl(n_bytes, t_ninf),
            "dq_quantize_pack_v": rl(M * dp * (4 + (b_last + 1) / 8), t_qv),
            "dq_unpack_dequant_reduce_v": rl(dp * (M * (b_last + 1) / 8 + 4), t_rv),
            "dq_unpack_dequant_reduce_v_per_worker": rl(dp * (M * (b_last + 1) / 8 + 4), t_rw),
            "dq_sign_pack": rl(M * dp * (4 + 1 / 8), t_sp),
            "dq_sign_reduce": rl(dp * (M / 8 + 4), t_sr),
            "dq_sign_majority": rl(dp * (M / 8 + 4), t_sm),
            "dq_sign_reduce_scaled": rl(dp * (M / 8 + 4), t_ss),
        },
    }
    # `traffic`: HBM bytes per launch (a number, like `achieved`'s numerator); where they come from beside it
    tr = profiled_traffic("k_quantize_pack")
    result["roofline"]["traffic"] = tr["bytes"] if tr else None
    result["roofline"]["traffic_detail"] = tr
    for entry, tag in (("dq_quantize_pack", "k_quantize_pack"), ("dq_unpack_dequant_reduce", "k_unpack_dequant_reduce"),
                       ("dq_norm", "k_norm_partial")):
        tk = profiled_traffic(tag)
        result["kernels"][entry]["traffic"] = tk["bytes"] if tk else None
    # step level: the two-call worker side reads every gradient twice (norm pass, quantize pass)
    result["step_traffic"] = {
        "algorithmic_bytes_per_step": int(n_bytes + q_bytes + r_bytes),
        "one_read_bytes_per_step": int(q_bytes + r_bytes),
        "traffic_vs_one_read": round((n_bytes + q_bytes + r_bytes) / (q_bytes + r_bytes), 4),
        "achieved_GBps": round((n_bytes + q_bytes + r_bytes) / (ms_per_step * 1e-3) / 1e9, 1),
        "note": "the single-pass entry points (bracketed_step, one_pass_step below) move one_read_bytes_per_step"}
    # f_Q of Eq. (7) for the timed steps: what the M workers would have put on the wire
    sent = sum(dq.comm_cost_bits(M, D, b, n_seg, 32) for b in bits)
    result["comm_cost"] = {"bits_sent": sent, "bits_uncompressed": len(bits) * dq.comm_cost_bits(M, D, 31, 0, 32),
                           "ratio": round(sent / (len(bits) * dq.comm_cost_bits(M, D, 31, 0, 32)), 5)}
    if one_pass is not None:
        t_fused, t_bred, ms_lagged, n_buckets = one_pass
        result["kernels"]["dq_norm_quantize_pack"] = rl(M * dp * (4 + (b_last + 1) / 8), t_fused)
        result["one_pass_step"] = {
            "what": "same gradient in 4096-element buckets (one norm each), b known beforehand (the paper's lagged "
                    "protocol): dq_norm_quantize_pack reads the gradient once, then dq_unpack_dequant_reduce",
            "buckets": n_buckets, "b": b_last, "ms_per_step": round(ms_lagged, 4),
            "value": round(in_bytes / (ms_lagged * 1e-3) / 1e9, 2), "unit": "GB/s of fp32 input",
            "reduce_ms": round(t_bred, 4)}
    result["kernels"]["dq_norm_quantize_pack_bracketed"] = rl(M * dp * (4 + (b_last + 1) / 8), t_br)
    result["bracketed_step"] = {
        "what": "the benchmark's own layout, b known beforehand, every norm known to +-12.5 % (the step before): "
                "dq_norm_quantize_pack_bracketed reads the gradient once, then dq_unpack_dequant_reduce",
        "b": b_last, "ms_per_step": round(ms_bracketed, 4),
        "value": round(in_bytes / (ms_bracketed * 1e-3) / 1e9, 2), "unit": "GB/s of fp32 input",
        "elements_settled_afterwards": br_counts[0], "chunks_quantized_again": br_counts[1]}
    result["lagged_one_pass_step"] = {
        "what": "Algorithm 1's protocol without a host round trip: widths on the GPU from the rule of the iteration "
                "before, dq_norm_quantize_pack_bracketed_v (norms known to +-12.5 %), dq_unpack_dequant_reduce_v, "
                "dq_select_bits_device for the next iteration",
        "ms_per_step": round(ms_lagged_device, 4), "value": round(in_bytes / (ms_lagged_device * 1e-3) / 1e9, 2),
        "unit": "GB/s of fp32 input"}
    result["device_rule_step"] = {
        "what": "the same step with dq_select_bits_device and the per-tensor-width kernels: no host round trip",
        "ms_per_step": round(ms_device_rule, 4), "value": round(in_bytes / (ms_device_rule * 1e-3) / 1e9, 2),
        "unit": "GB/s of fp32 input"}
    # what library kernels (not this repository's) reach on the same buffers at several read/write mixes
    # (large workloads only: below 256 MiB the data sits in the Infinity Cache)
    if M * dp * 4 >= (1 << 28):
        indep = independent_ceiling()
        if indep:
            result["independent_ceiling"] = {
                "what": "GB/s (read + written) of torch / HIP-runtime kernels on this run's buffers, timed with the same "
                        "events; the 4:1 and 4:2 conversions bracket quantize+pack's mix (4 : (b+1)/8), the 2:4 and "
                        "4:4 ones the reduce's (M(b+1)/8 : 4)",
                "kernels": indep}
            lt = next(v for k, v in indep.items() if k.startswith("fp32 -> bool"))["GBps"]
            h2f = next(v for k, v in indep.items() if k.startswith("fp32 -> fp16"))["GBps"]
            result["kernels"]["dq_quantize_pack"]["frac_of_independent_4to1"] = round(result["kernels"]["dq_quantize_pack"]["achieved"] / lt, 4)
            result["kernels"]["dq_unpack_dequant_reduce"]["frac_of_independent_4to2"] = round(result["kernels"]["dq_unpack_dequant_reduce"]["achieved"] / h2f, 4)
            result["roofline"]["frac_of_independent_4to1"] = result["kernels"]["dq_quantize_pack"]["frac_of_independent_4to1"]
    # both fused passes at every level width b = 1..8 on the same gradients (not part of `value`):
    # time, algorithmic GB/s and fraction of the HBM peak
    per_b = {}
    for b in range(1, 9):
        pk_b = packed[:, :plan.packed_bytes(b)]
        # three untimed calls first: whichever width runs first after the host-side pause before this
        # sweep otherwise measures 5 % slow (clocks still rising), whatever that width is
        tq = timed_loop(lambda: dq.quantize_pack(plan, grads, norms_dev, b, wl.QUANT_SEED, T, pk_b), 4, warm=3 if b == 1 else 1)
        tr = timed_loop(lambda: dq.unpack_dequant_reduce(plan, pk_b, norms_dev, b, out), 4)
        q, r = rl(M * dp * (4 + (b + 1) / 8), tq), rl(dp * (M * (b + 1) / 8 + 4), tr)
        row = {"quantize_pack_ms": q["avg_ms"], "quantize_pack_GBps": q["achieved"], "quantize_pack_frac": q["frac"],
               "reduce_ms": r["avg_ms"], "reduce_GBps": r["achieved"], "reduce_frac": r["frac"]}
        per_b[str(b)] = row
    result["per_b"] = per_b
    # put the messages and the average of the last timed step back
    dq.quantize_pack(plan, grads, norms_dev, b_last, wl.QUANT_SEED, T - 1, pk_last)
    dq.unpack_dequant_reduce(plan, pk_last, norms_dev, b_last, out)
    torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        b_mode = max(set(bits), key=bits.count)
        result["cpu_baseline"] = cpu_baseline(seg_len, grads, b_mode, 1 << args.cpu_sample_log2,
                                                  max(1, args.cpu_steps))
    print(json.dumps(result), flush=True)
    plan.close()


if __name__ == "__main__":
    main()
