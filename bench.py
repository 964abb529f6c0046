"""Benchmark of the CafeQ hot path on one MI355X.

Headline workload: the Gemma-2-9B-shaped MLP pair (down 3584x14336 gets T on its columns, up 14336x3584 gets
T^-1 on its rows), block-diagonal 128x128 transform, 3-bit symmetric absmax grid, group 128 -- synthetic
Student-t weights with outliers (workloads.config3).  One step = one evaluation of the whole path as the
paper's learning loop runs it: blockwise inverse of the transform, then the paired proxy-loss forward +
backward (transform, group absmax, RTN codes, dequantize, inverse transform, error reductions, LogSumExp
surrogate and its gradient w.r.t. T).  All inputs are resident in HBM before the timed region; the weights,
which are constant over a learning run, are also held in the library's prepared form
(cafeq_prepare_weights, once, outside the timed region; its cost is reported).

Prints ONE JSON line: weight-elements/s over the whole job; the roofline of the dominant kernel (the loss
pass), its duration measured with HIP events recorded on the launch stream around every launch inside the
timed region; the CPU oracle timed on the host cores on a bounded sample; and a `secondary` list with the
same step under other conditions (a transform part-way through learning, whose inverse takes the elimination
kernel; the unprepared path) and the other workloads (plain quantizer, single matrix, Alg. 1, the 27B-shaped
layer).  `--workload NAME` prints the line of one secondary workload alone.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

F16_MFMA_PEAK_TFLOPS = 2500.0
FP32_MFMA_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0


def memory_probe(torch, dev, cafeq):
    """Streaming rates over 1 GiB buffers (larger than every cache of the part): the library's own plain streaming
    read (cafeq_stream_read_probe: what the memory system delivers to a kernel that only reads), and, for
    comparison, two of torch's kernels (a read-only reduction and a copy).  Context for the roofline figures, not
    part of any timed step."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)

    def rate(fn, nbytes, n=10):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return nbytes * n / (time.perf_counter() - t0) / 1e12

    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    out = {"read_only_TBps": rate(lambda: cafeq.stream_read_probe(src, sink), src.numel() * 4),
           "torch_sum_TBps": rate(lambda: src.sum(), src.numel() * 4),
           "torch_copy_read_plus_write_TBps": rate(lambda: dst.copy_(src), 2 * src.numel() * 4),
           "what": "cafeq_stream_read_probe / torch.sum / Tensor.copy_ over 1 GiB float32, 10 repetitions"}
    del src, dst
    torch.cuda.empty_cache()
    return out


def measured_traffic(profile, key):
    """HBM bytes per launch from a rocprofv3 summary under profiles/ (a line `key: <bytes>`), or None."""
    try:
        text = open(os.path.join(ROOT, "profiles", profile)).read()
    except OSError:
        return None
    m = re.search(r"^%s:\s*([0-9.eE+]+)" % re.escape(key), text, flags=re.M)
    return float(m.group(1)) if m else None


def _cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return os.cpu_count() or 1


def _base(metric, value, unit, steps, warmup, ms, dtype, workload, **cfg):
    return {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype,
            "data": "synthetic", "config": dict(workload=workload, **cfg)}


def _timed(torch, fn, steps, warmup):
    for _ in range(max(warmup, 1)):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


# ----------------------------------------------------------------------------------------------------
# headline: the 9B-shaped pair
# ----------------------------------------------------------------------------------------------------
def pair_cpu_baseline(cfg, blocks, reps):
    """The oracle as it stands, on the first `blocks` transform blocks of the pair."""
    import numpy as np
    from oracle import cafeq_oracle as O
    k = cfg["k"]
    A = np.ascontiguousarray(cfg["A"][:, :blocks * k])
    B = np.ascontiguousarray(cfg["B"][:blocks * k, :])
    T = cfg["T"][:blocks]
    t0 = time.perf_counter()
    for _ in range(reps):
        P = O.block_inverse(T)
        O.dual_lse(A, B, T, P, cfg["bits"][0], cfg["group"], cfg["rep"], 5.0)
    dt = time.perf_counter() - t0
    elems = A.size + B.size
    return {"value": elems * reps / dt, "unit": "weight-elements/s", "cores": _cores(), "kind": "oracle",
            "sample": "%d of %d transform blocks of the same pair (%.1f M weights), %d x (block inverse + "
                      "fwd+bwd), %.1f s" % (blocks, cfg["T"].shape[0], elems / 1e6, reps, dt)}


def pair_workload(args, secondary=True):
    import numpy as np
    import torch
    from paper_2511_19705_amd import cafeq, workloads as WL
    dev = torch.device("cuda:0")
    cfg = WL.config3()
    k, g, bits, rep = cfg["k"], cfg["group"], cfg["bits"][0], cfg["rep"]
    A = torch.from_numpy(cfg["A"]).to(dev)
    B = torch.from_numpy(cfg["B"]).to(dev)
    T = torch.from_numpy(cfg["T"]).to(dev)
    elems = A.numel() + B.numel()
    member = elems / 2.0

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 1 GiB, writes 1 GiB: reference for the profiler's byte counters
        torch.cuda.synchronize()
        del src, dst

    # the weights in the library's prepared form: once per learning run
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    prep = (cafeq.prepare_weights(A, cafeq.AXIS_COL), cafeq.prepare_weights(B, cafeq.AXIS_ROW))
    torch.cuda.synchronize()
    prep_ms = (time.perf_counter() - t0) * 1e3

    def make_step(Tx, prepared):
        def step():
            P, _ = cafeq.block_inverse(Tx)
            return cafeq.dual_proxy_loss_fwd_bwd(A, B, Tx, P, bits, g, rep, 5.0, want_grad=True, prepared=prepared)
        return step

    step = make_step(T, prep)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # every fifth launch of the loss pass is timed (members alternate): an event pair holds the stream up for
    # several microseconds, which would otherwise be part of every step
    timer = cafeq.LaunchTimer(2 * args.steps // 5 + 2, every=5)   # (one or two launches per step)
    with timer:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    durs = timer.durations_ms()
    losses = out[0].cpu().numpy()

    # dominant kernel: the loss pass, launched once per member.  Algorithmic work per launch: forward and inverse
    # transform of its member, 2k flop per element each; it reads every weight once (4 B per element).
    # (with prepared weights and no codes requested the library runs both members' loss passes as ONE launch, each
    # member on half of the chip: the timing table says how many launches there were)
    launches_per_step = max(1, round(timer.table.seen / float(args.steps)))
    per_launch = member * (2.0 / launches_per_step)           # weight elements one launch covers
    avg_launch_s = sum(durs) / max(len(durs), 1) * 1e-3
    flops_per_launch = 2.0 * 2.0 * k * per_launch
    achieved = flops_per_launch / avg_launch_s / 1e12
    executed = 5.0 * 2.0 * k * per_launch / avg_launch_s / 1e12   # 3 + 2 part products per contraction index
    result = _base("proxy-loss fwd+bwd weight-elements/s (9B-shaped MLP pair, dual transform)", elems * args.steps / dt,
                   "weight-elements/s", args.steps, args.warmup, dt / args.steps * 1e3, "f32", cfg["name"],
                   rows_cols=[list(cfg["A"].shape), list(cfg["B"].shape)], block=k, group=g, bits=bits,
                   evals_per_s=args.steps / dt,
                   step="block inverse + dual proxy-loss fwd+bwd (a loss pass per member, one gradient pass over both)",
                   weights="resident in HBM, also in prepared form (cafeq_prepare_weights once per learning run, "
                           "%.2f ms for both members, outside the timed region)" % prep_ms,
                   inverse="T is the workload's rotation (the paper's initialisation): blocks verified to be rotations are "
                           "inverted by transposition; see secondary[c3_pair_midlearning] for any other transform",
                   contraction="forward: 2 float16 parts per operand, 3 products; inverse: float16 error x 2 float16 parts, "
                               "2 products; float32 accumulate",
                   relative_l2_A=float((losses[2] / float((cfg["A"].astype("float64") ** 2).sum())) ** 0.5))
    # The loss pass does 4k = 512 flop per 4 bytes it has to read: 128 flop/B, below the part's 2500 TFLOP/s :
    # 8 TB/s = 312 flop/B, so the roofline that bounds it is the memory one.  (The matrix-pipe figures stay in the
    # object: "mfma".)
    hbm_gbs = 4.0 * per_launch / avg_launch_s / 1e9
    result["roofline"] = {
        "bound": "hbm", "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS,
        "traffic": measured_traffic("loss_prepared_c3_pair.md", "traffic_bytes_per_launch"),
        "kernel": "loss_v2_pair_kernel<128,true> (loss pass over prepared weights, both members of the pair in one "
                  "launch)" if launches_per_step == 1 else "loss_v2_kernel<128,*,true,false> (loss pass over prepared weights)",
        "launches": len(durs), "launches_in_timed_region": int(timer.table.seen),
        "weight_elements_per_launch": per_launch,
        "avg_launch_us": avg_launch_s * 1e6, "algorithmic_flop_per_element": 4 * k,
        "algorithmic_bytes_per_element": 4,
        "arithmetic_intensity_flop_per_byte": k, "ridge_flop_per_byte": F16_MFMA_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBS,
        "mfma": {"achieved": achieved, "peak": F16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": achieved / F16_MFMA_PEAK_TFLOPS, "executed_part_product_tflops": executed,
                 "executed_frac_of_f16_peak": executed / F16_MFMA_PEAK_TFLOPS,
                 "achieved_over_fp32_mfma_peak": achieved / FP32_MFMA_PEAK_TFLOPS},
        "whole_step_hbm_frac_at_one_read_of_the_weights": 4.0 * elems * args.steps / dt / 1e9 / HBM_PEAK_GBS}
    # the step's other large kernel, timed the same way in a short loop of its own (one table times one kind of
    # launch): the gradient pass reads both members' second prepared copy once, 4 B per element
    gsteps = max(10, min(args.steps, 50))
    gtimer = cafeq.LaunchTimer(gsteps // 5 + 2, every=5, kind=1)
    with gtimer:
        for _ in range(gsteps):
            step()
        torch.cuda.synchronize()
    gd = gtimer.durations_ms()
    if gd:
        g_s = sum(gd) / len(gd) * 1e-3
        g_launches = max(1, round(gtimer.table.seen / float(gsteps)))
        g_el = elems / g_launches
        result["roofline_gradient_pass"] = {
            "bound": "hbm", "achieved": 4.0 * g_el / g_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": 4.0 * g_el / g_s / 1e9 / HBM_PEAK_GBS,
            "traffic": measured_traffic("loss_prepared_c3_pair.md", "gradient_traffic_bytes_per_launch"),
            "kernel": "grad_v2_owner_kernel (gradient pass over prepared weights, one workgroup per member and block)",
            "launches": len(gd), "launches_in_timed_region": int(gtimer.table.seen),
            "weight_elements_per_launch": g_el, "avg_launch_us": g_s * 1e6,
            "algorithmic_bytes_per_element": 4, "algorithmic_flop_per_element": 2 * k,
            "executed_part_product_tflops": 3.0 * 2.0 * k * g_el / g_s / 1e12}
    # what this machine's memory system delivers to plain streaming kernels on data that no cache holds (the published
    # 8 TB/s stays the roofline's peak; these two figures say how far any kernel gets towards it here)
    probe = memory_probe(torch, dev, cafeq)
    traffic = result["roofline"]["traffic"]
    result["roofline"]["memory_probe"] = probe
    if traffic:
        result["roofline"]["measured_traffic_TBps"] = traffic / avg_launch_s / 1e12
        result["roofline"]["measured_traffic_over_read_probe"] = traffic / avg_launch_s / 1e12 / probe["read_only_TBps"]
    if secondary:
        sec = []
        n2 = max(10, args.steps // 4)
        # the same step with a transform part-way through learning: every block goes through the elimination
        Tm = torch.from_numpy(WL.perturbed_blocks(cfg["T"].shape[0], k, 304, 0.05)).to(dev)
        d2 = _timed(torch, make_step(Tm, prep), n2, 3)
        sec.append({"workload": "c3_pair_midlearning", "what": "same step, T = rotation x (I + 0.05 G / sqrt(k)): inverse by "
                    "elimination", "steps": n2, "ms_per_step": d2 / n2 * 1e3, "value": elems * n2 / d2, "unit": "weight-elements/s"})
        d3 = _timed(torch, make_step(T, (None, None)), n2, 3)
        sec.append({"workload": "c3_pair_unprepared", "what": "same step without prepared weights (float32 weights split per "
                    "call)", "steps": n2, "ms_per_step": d3 / n2 * 1e3, "value": elems * n2 / d3, "unit": "weight-elements/s"})
        del prep, A, B
        torch.cuda.empty_cache()
        sub = argparse.Namespace(**vars(args))
        sub.no_cpu_baseline = True
        sub.steps, sub.warmup = n2, 3
        for name in ("c3_rtn", "c3_optimize", "c2_single", "c4_dual", "c4_optimize", "c4_adaptive", "c5_layer"):
            sub.workload = name
            r = WORKLOADS[name](sub)
            sec.append({"workload": r["config"]["workload"], "metric": r["metric"], "steps": r["steps"],
                        "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": r["unit"],
                        "roofline": {kk: r["roofline"][kk] for kk in ("bound", "achieved", "peak", "unit", "frac", "kernel")
                                     if kk in r.get("roofline", {})},
                        **({"detail": r["detail"]} if "detail" in r else {})})
            torch.cuda.empty_cache()
        result["secondary"] = sec
    # (the oracle on the host cores comes last: its thread pools keep spinning for a while after a run, and the
    # secondary workloads with many small launches per step are then starved by the launching thread's neighbours)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = pair_cpu_baseline(cfg, args.cpu_blocks, args.cpu_reps)
    return result


# ----------------------------------------------------------------------------------------------------
# secondary workloads
# ----------------------------------------------------------------------------------------------------
def core_workload(args):
    """c3_optimize : Adam iterations on the 9B-shaped pair (inverse + paired fwd+bwd + update), prepared weights
       c2_single   : single-matrix fwd+bwd on the 2B-shaped down projection (k = 64, fused gradient)
       c4_adaptive : Alg. 1 iterations on the 9B-shaped attention V/O pair (k = 256)"""
    import numpy as np
    import torch
    from paper_2511_19705_amd import cafeq, workloads as WL
    dev = torch.device("cuda:0")
    if args.workload == "c3_optimize":
        cfg = WL.config3()
        A, B = torch.from_numpy(cfg["A"]).to(dev), torch.from_numpy(cfg["B"]).to(dev)
        T = torch.from_numpy(cfg["T"].copy()).to(dev)
        prep = (cafeq.prepare_weights(A, 0), cafeq.prepare_weights(B, 1))
        elems, k = A.numel() + B.numel(), cfg["k"]
        run = lambda n: cafeq.optimize_pair(A, B, T, cfg["bits"][0], cfg["group"], 1, 5.0, 1e-3, n, prepared=prep)
        metric = "learning iterations, weight-elements/s (Adam on the LogSumExp surrogate, 9B-shaped MLP pair)"
        flop_el, parts, kern, name = 4 * k, 5, "loss_v2_pair_kernel<128,true> (loss pass, both members in one launch)", cfg["name"] + "_adam"

        def cpu():
            from oracle import cafeq_oracle as O
            nbk = 16
            a = np.ascontiguousarray(cfg["A"][:, :nbk * k]); b = np.ascontiguousarray(cfg["B"][:nbk * k, :])
            t0 = time.perf_counter()
            O.optimize_pair(a, b, cfg["T"][:nbk], cfg["bits"][0], cfg["group"], 1, 5.0, 1e-3, 2)
            dt = time.perf_counter() - t0
            return (a.size + b.size) * 2 / dt, "%d of %d blocks of the pair, 2 Adam iterations, %.1f s" % (nbk, cfg["T"].shape[0], dt)
    elif args.workload == "c2_single":
        cfg = WL.config2()
        W = torch.from_numpy(cfg["W"]).to(dev)
        T = torch.from_numpy(cfg["T"]).to(dev)
        elems, k = W.numel(), cfg["k"]

        def run(n):
            for _ in range(n):
                P, _ = cafeq.block_inverse(T)
                cafeq.proxy_loss_fwd_bwd(W, T, P, cfg["bits"][0], cfg["group"], 0, 1, want_grad=True)
        metric = "proxy-loss fwd+bwd weight-elements/s (2B-shaped down projection, single transform)"
        flop_el, parts, kern, name = 6 * k, 12, "xform_core_kernel<64,128,COL,true> (fused)", cfg["name"]

        def cpu():
            from oracle import cafeq_oracle as O
            nbk = 48
            w = np.ascontiguousarray(cfg["W"][:, :nbk * k]); t = cfg["T"][:nbk]
            t0 = time.perf_counter()
            for _ in range(3):
                p_ = O.block_inverse(t)
                O.proxy_l2(w, t, p_, cfg["bits"][0], cfg["group"], 0, 1)
                O.surrogate(w, t, p_, cfg["bits"][0], cfg["group"], 0, 1)
            dt = time.perf_counter() - t0
            return w.size * 3 / dt, "%d of %d blocks, 3 x (inverse + fwd+bwd), %.1f s" % (nbk, cfg["T"].shape[0], dt)
    elif args.workload == "c4_optimize":
        # Adam iterations on the attention pair at the paper's 9B block size (inverse warm-started by Newton-Schulz rounds)
        cfg = WL.config4()
        k, rep, g, bits = cfg["k"], cfg["rep"], cfg["group"], cfg["bits"][0]
        A, B = torch.from_numpy(cfg["A"]).to(dev), torch.from_numpy(cfg["B"]).to(dev)
        T = torch.from_numpy(cfg["T"].copy()).to(dev)
        elems = A.numel() + B.numel()
        run = lambda n: cafeq.optimize_pair(A, B, T, bits, g, rep, 5.0, 1e-3, n)
        metric = "learning iterations, weight-elements/s (Adam on the LogSumExp surrogate, 9B-shaped attention V/O pair, blocks of 256)"
        flop_el, parts, kern, name = 4 * k, 9, "xform_core_kernel<256,64,*,false,true> (loss pass)", cfg["name"] + "_adam"

        def cpu():
            from oracle import cafeq_oracle as O
            nh = 2
            a = np.ascontiguousarray(cfg["A"][:, :nh * k]); b = np.ascontiguousarray(cfg["B"][:nh * rep * k, :])
            t0 = time.perf_counter()
            O.optimize_pair(a, b, cfg["T"][:nh], bits, g, rep, 5.0, 1e-3, 1)
            dt = time.perf_counter() - t0
            return (a.size + b.size) / dt, "%d of %d heads, 1 Adam iteration, %.1f s" % (nh, cfg["T"].shape[0], dt)
    elif args.workload == "c4_dual":
        # the paired loss and gradient at the block size the paper runs the 9B model with (per-head 256 x 256, kv heads
        # shared by two query heads): block inverse + cafeq_dual_proxy_loss_fwd_bwd with gradient
        cfg = WL.config4()
        k, rep, g, bits = cfg["k"], cfg["rep"], cfg["group"], cfg["bits"][0]
        A, B = torch.from_numpy(cfg["A"]).to(dev), torch.from_numpy(cfg["B"]).to(dev)
        T = torch.from_numpy(cfg["T"]).to(dev)
        elems = A.numel() + B.numel()

        def run(n):
            for _ in range(n):
                P, _ = cafeq.block_inverse(T)
                cafeq.dual_proxy_loss_fwd_bwd(A, B, T, P, bits, g, rep, 5.0, want_grad=True)
        metric = "proxy-loss fwd+bwd weight-elements/s (9B-shaped attention V/O pair, per-head 256 x 256 dual transform)"
        flop_el, parts, kern, name = 4 * k, 9, "xform_core_kernel<256,64,*,false,true> (loss pass)", cfg["name"] + "_dual"

        def cpu():
            from oracle import cafeq_oracle as O
            nh = 2
            a = np.ascontiguousarray(cfg["A"][:, :nh * k]); b = np.ascontiguousarray(cfg["B"][:nh * rep * k, :])
            t = cfg["T"][:nh]
            t0 = time.perf_counter()
            p_ = O.block_inverse(t)
            O.dual_lse(a, b, t, p_, bits, g, rep, 5.0)
            dt = time.perf_counter() - t0
            return (a.size + b.size) / dt, "%d of %d heads, 1 x (inverse + fwd+bwd), %.1f s" % (nh, cfg["T"].shape[0], dt)
    else:
        cfg = WL.config4()
        k, rep, g, bits = cfg["k"], cfg["rep"], cfg["group"], cfg["bits"][0]
        A, B = torch.from_numpy(cfg["A"]).to(dev), torch.from_numpy(cfg["B"]).to(dev)
        T = torch.from_numpy(cfg["T"]).to(dev)
        P, _ = cafeq.block_inverse(T)
        U = cafeq.apply_transform(A, T, P, 0, cafeq.SIDE_T, 1)
        V = cafeq.apply_transform(B, T, P, 1, cafeq.SIDE_TINV, rep)
        cu, su, _ = cafeq.rtn_quantize(U, bits, g, 0)
        cv, sv, _ = cafeq.rtn_quantize(V, bits, g, 1)
        elems = U.numel() + V.numel()

        def run(n):
            for _ in range(n):
                cafeq.adaptive_round_step(U, V, cu, su, cv, sv, bits, g, k, rep, half=0)
        metric = "adaptive-rounding iterations, weight-elements/s (Alg. 1, 9B-shaped attention V/O pair)"
        flop_el, parts, kern, name = 2 * k, 6, "xform_core_kernel<256,64,*,false> (transform + requantize)", cfg["name"]

        def cpu():
            from oracle import cafeq_oracle as O
            Un, Vn = U.cpu().numpy(), V.cpu().numpy()
            nh = 2
            u = np.ascontiguousarray(Un[:, :nh * k]); v = np.ascontiguousarray(Vn[:nh * rep * k, :])
            c0, s0, _ = O.rtn_sym(u, bits, g, O.COL)
            uh = c0.astype(np.float64) * np.repeat(s0.astype(np.float64), g, axis=1)
            t0 = time.perf_counter()
            O.adaptive_round_step(u, v, uh, bits, g, k, rep)
            dt = time.perf_counter() - t0
            return (u.size + v.size) / dt, "%d of %d heads, 1 iteration (SVD pseudoinverse), %.1f s" % (nh, cfg["T"].shape[0], dt)

    run(max(args.warmup, 1))
    torch.cuda.synchronize()
    timer = cafeq.LaunchTimer(8 * args.steps + 8, every=5)
    with timer:
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    durs = timer.durations_ms()
    avg = sum(durs) / max(len(durs), 1) * 1e-3
    # (weight elements one timed launch covers: the timing table counts every eligible launch, timed or not)
    per_launch_el = elems * args.steps / max(int(timer.table.seen), 1)
    achieved = flop_el * per_launch_el / avg / 1e12
    out = _base(metric, elems * args.steps / dt, "weight-elements/s", args.steps, args.warmup, dt / args.steps * 1e3,
                "f32", name, block=cfg["k"], group=cfg["group"], bits=cfg["bits"][0])
    out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": F16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": achieved / F16_MFMA_PEAK_TFLOPS, "traffic": None, "kernel": kern, "launches": len(durs),
                       "launches_in_timed_region": int(timer.table.seen),
                       "avg_launch_us": avg * 1e6, "algorithmic_flop_per_element": flop_el,
                       "executed_part_product_tflops": achieved * parts * 2 * cfg["k"] / flop_el}
    if not args.no_cpu_baseline:
        v, sample = cpu()
        out["cpu_baseline"] = {"value": v, "unit": "weight-elements/s", "cores": _cores(), "kind": "oracle", "sample": sample}
    return out


def layer_workload(args):
    """The 27B-shaped decoder layer, bfloat16 storage, k = 128, group 128: per bit-width (3 and 4), the proxy-loss
    forward + backward of every single (q, k, gate) and pair ((down, up), (V, O)) -- one evaluation each, as one
    iteration of the learning loops -- followed by the final quantization of all seven matrices (codes and scales
    written).  One step = that sequence for both bit-widths; the layer wall time per bit-width is in `detail`."""
    import numpy as np
    import torch
    from paper_2511_19705_amd import cafeq, workloads as WL
    dev = torch.device("cuda:0")
    meta = WL.config5_meta()
    k, g, rep = meta["k"], meta["group"], meta["rep"]
    host = {nm: WL.config5_tensor(nm) for nm in ("q", "k", "gate", "down", "up", "v", "o")}
    Wd = {nm: torch.from_numpy(t["bits16"].view(np.int16)).to(dev).view(torch.bfloat16) for nm, t in host.items()}
    Ts = {w: torch.from_numpy(WL.config5_transform(w)).to(dev) for w in ("single", "mlp", "vo")}
    axis = {"q": 0, "k": 0, "gate": 0, "down": 0, "up": 1, "v": 0, "o": 1}
    prep = {nm: cafeq.prepare_weights(Wd[nm], axis[nm]) for nm in Wd}
    elems = sum(w.numel() for w in Wd.values())

    def evaluate(bits):
        Ps, _ = cafeq.block_inverse(Ts["single"])
        for nm in ("q", "k", "gate"):
            cafeq.proxy_loss_fwd_bwd(Wd[nm], Ts["single"], Ps, bits, g, 0, 1, want_grad=True, prepared=prep[nm])
        Pm, _ = cafeq.block_inverse(Ts["mlp"])
        cafeq.dual_proxy_loss_fwd_bwd(Wd["down"], Wd["up"], Ts["mlp"], Pm, bits, g, 1, 5.0, want_grad=True,
                                      prepared=(prep["down"], prep["up"]))
        Pv, _ = cafeq.block_inverse(Ts["vo"])
        cafeq.dual_proxy_loss_fwd_bwd(Wd["v"], Wd["o"], Ts["vo"], Pv, bits, g, rep, 5.0, want_grad=True,
                                      prepared=(prep["v"], prep["o"]))
        return Ps, Pm, Pv

    def finalize(bits, Ps, Pm, Pv):
        for nm in ("q", "k", "gate"):
            cafeq.proxy_loss_fwd_bwd(Wd[nm], Ts["single"], Ps, bits, g, 0, 1, want_grad=False, want_codes=True,
                                     prepared=prep[nm])
        cafeq.dual_proxy_loss_fwd_bwd(Wd["down"], Wd["up"], Ts["mlp"], Pm, bits, g, 1, 5.0, want_grad=False,
                                      want_codes=True, prepared=(prep["down"], prep["up"]))
        cafeq.dual_proxy_loss_fwd_bwd(Wd["v"], Wd["o"], Ts["vo"], Pv, bits, g, rep, 5.0, want_grad=False,
                                      want_codes=True, prepared=(prep["v"], prep["o"]))

    per_bits = {}
    for bits in meta["bits"]:
        inv = evaluate(bits)
        finalize(bits, *inv)
    torch.cuda.synchronize()
    steps = max(3, args.steps // 4)
    t_all = 0.0
    for bits in meta["bits"]:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            inv = evaluate(bits)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            finalize(bits, *inv)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        per_bits["%d_bit" % bits] = {"fwd_bwd_ms": (t1 - t0) / steps * 1e3, "final_quantize_ms": (t2 - t1) / steps * 1e3,
                                     "layer_ms": (t2 - t0) / steps * 1e3}
        t_all += t2 - t0
    passes = 2 * len(meta["bits"])              # every weight is read by one fwd+bwd and one final quantization per bit-width
    out = _base("layer quantization wall time, weight-elements/s (27B-shaped decoder layer: fwd+bwd of q, k, gate, "
                "(down, up), (V, O) and final quantization of all seven, 3 and 4 bit)", elems * passes * steps / t_all,
                "weight-elements/s", steps, 1, t_all / steps * 1e3, "f32 (bf16 storage)",
                "c5_27b_layer_bf16_k%d_g%d_b3_b4" % (k, g), block=k, group=g, bits=list(meta["bits"]))
    out["detail"] = per_bits
    out["roofline"] = {"bound": "mfma", "achieved": None, "peak": F16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": None,
                       "traffic": None, "kernel": "loss_v2_kernel<128,*,*,*> (bfloat16-stored weights, prepared)"}
    if not args.no_cpu_baseline:
        from oracle import cafeq_oracle as O
        w = WL.bf16_bits_to_f32(host["q"]["bits16"])
        t = WL.config5_transform("single")
        t0 = time.perf_counter()
        for _ in range(4):
            p_ = O.block_inverse(t)
            O.proxy_l2(w, t, p_, 3, g, 0, 1)
            O.surrogate(w, t, p_, 3, g, 0, 1)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": w.size * 4 / dt, "unit": "weight-elements/s", "cores": _cores(), "kind": "oracle",
                               "sample": "the q projection (4096 x 4608, 36 blocks), 4 x (inverse + fwd+bwd), %.1f s" % dt}
    return out


def infer_workload(args):
    """Inference side of a single transformed matrix (Sec. 4.1; the block-size table's extra wall-clock row):
    one token through the quantized down projection, with and without the inverse transform on the
    activations.  c2_infer: the table's matrix (in 9216, out 2304); c3_infer: the 9B-shaped one (in 14336,
    out 3584).  Codes and scales are synthetic (the entry point sees nothing else of the weight)."""
    import numpy as np
    import torch
    from paper_2511_19705_amd import cafeq
    dev = torch.device("cuda:0")
    out_f, in_f = (2304, 9216) if args.workload == "c2_infer" else (3584, 14336)
    k, g, bits, n = 128, 128, 4, 1
    gen = torch.Generator(device="cpu").manual_seed(77)
    codes_h = torch.randint(-8, 8, (out_f, in_f), dtype=torch.int8, generator=gen)
    scales_h = torch.exp(torch.randn((out_f, in_f // g), generator=gen) * 0.5 - 5.0)
    P_h = torch.eye(k).repeat(in_f // k, 1, 1) + 0.05 * torch.randn((in_f // k, k, k), generator=gen) / k ** 0.5
    X_h = torch.randn((n, in_f), generator=gen)
    codes, scales, P, X = codes_h.to(dev), scales_h.to(dev), P_h.to(dev), X_h.to(dev)
    Y = torch.empty((n, out_f), device=dev)

    def timed(fn, reps):
        for _ in range(max(args.warmup, 1)):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3, (time.perf_counter() - t0) / reps

    plain_ev, _ = timed(lambda: cafeq.infer_single(X, None, codes, scales, g, out=Y), args.steps)
    xf_ev, xf_wall = timed(lambda: cafeq.infer_single(X, P, codes, scales, g, out=Y), args.steps)
    byts = out_f * in_f + out_f * (in_f // g) * 4 + n * in_f * 4 + n * out_f * 4
    achieved = byts / plain_ev / 1e9
    res = _base("tokens/s through one quantized transformed layer (activation transform + dequantize + product)",
                n / xf_wall, "tokens/s", args.steps, args.warmup, xf_wall * 1e3, "f32",
                "%s_%dx%d_k%d_g%d_%dbit_tokens%d" % (args.workload, out_f, in_f, k, g, bits, n))
    res["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                       "traffic": None, "kernel": "dequant_gemv_kernel<1,*> (plain quantized layer)",
                       "avg_launch_us": plain_ev * 1e6, "algorithmic_bytes": byts}
    res["transform"] = {"plain_us": plain_ev * 1e6, "with_transform_us": xf_ev * 1e6,
                        "extra_wall_clock_pct": (xf_ev / plain_ev - 1) * 100,
                        "extra_flops_pct": 100.0 * k / out_f, "extra_bytes_pct": 100.0 * 4 * k / out_f}
    if not args.no_cpu_baseline:
        from oracle import cafeq_oracle as O
        rows = 256
        c, sc = codes_h[:rows].numpy(), scales_h[:rows].numpy()
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            O.infer_single(X_h.numpy(), P_h.numpy(), c, sc, g)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        res["cpu_baseline"] = {"value": n / (dt * out_f / rows), "unit": "tokens/s", "cores": _cores(), "kind": "oracle",
                               "sample": "%d of %d output rows (dense inverse transform included), %d repetitions, scaled" % (rows, out_f, reps)}
    return res


def rtn_workload(args):
    """Plain per-group round-to-nearest (no transform) of the first member of the 9B-shaped pair ([3584][14336],
    groups of 128 along the contiguous axis): the HBM-bound stage of the path.
    Algorithmic bytes per element: 4 read + 1 code + 4/g scale."""
    import torch
    from paper_2511_19705_amd import cafeq, workloads as WL
    dev = torch.device("cuda:0")
    cfg = WL.config3()
    W = torch.from_numpy(cfg["A"]).to(dev)
    g, bits = cfg["group"], cfg["bits"][0]
    elems = W.numel()
    run = lambda: cafeq.rtn_quantize(W, bits, g, 0)
    for _ in range(max(args.warmup, 1)):
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern_s = e0.elapsed_time(e1) / args.steps * 1e-3
    byts = elems * (4 + 1 + 4.0 / g)
    achieved = byts / kern_s / 1e9
    res = _base("round-to-nearest weight-elements/s (9B-shaped projection, no transform)", elems * args.steps / dt,
                "weight-elements/s", args.steps, args.warmup, dt / args.steps * 1e3, "f32",
                "c3_rtn_3584x14336_g%d_b%d" % (g, bits), group=g, bits=bits)
    res["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                       "traffic": measured_traffic("rtn_col_fast_c3_member.md", "traffic_bytes_per_launch"),
                       "kernel": "rtn_col_fast<F32Tag, 32>", "avg_launch_us": kern_s * 1e6,
                       "algorithmic_bytes_per_element": 4 + 1 + 4.0 / g}
    if not args.no_cpu_baseline:
        from oracle import cafeq_oracle as O
        rows = 512
        w = cfg["A"][:rows]
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            O.rtn_sym(w, bits, g, O.COL)
            reps += 1
        dtc = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": w.size * reps / dtc, "unit": "weight-elements/s", "cores": _cores(), "kind": "oracle",
                               "sample": "%d of %d rows, %d repetitions, %.1f s" % (rows, cfg["A"].shape[0], reps, dtc)}
    return res


WORKLOADS = {"c3_optimize": core_workload, "c2_single": core_workload, "c4_adaptive": core_workload, "c4_dual": core_workload,
             "c4_optimize": core_workload,
             "c5_layer": layer_workload, "c2_infer": infer_workload, "c3_infer": infer_workload, "c3_rtn": rtn_workload}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="headline only (no secondary list)")
    ap.add_argument("--cpu-blocks", type=int, default=112)
    ap.add_argument("--cpu-reps", type=int, default=4)
    ap.add_argument("--workload", default="c3_pair", choices=["c3_pair"] + sorted(WORKLOADS),
                    help="c3_pair is the headline metric; the others are secondary measurements")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (the path is sharded by transform block "
                 "in design only); --gpus %d is not available" % args.gpus)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "c3_pair":
        res = pair_workload(args, secondary=not args.no_secondary)
    else:
        res = WORKLOADS[args.workload](args)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
