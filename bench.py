"""Benchmark of the CafeQ hot path on one MI355X.

Workload (default): the Gemma-2-9B-shaped MLP pair (down 3584x14336 gets T on its columns,
up 14336x3584 gets T^-1 on its rows), block-diagonal 128x128 transform, 3-bit symmetric
absmax grid, group 128 -- synthetic Student-t weights with outliers (workloads.config3).
One step = one evaluation of the whole path: blockwise inverse of the transform, then the
paired proxy-loss forward + backward (transform, group absmax, RTN codes, dequantize,
inverse transform, error reductions, LogSumExp surrogate and its gradient w.r.t. T).
Inputs are resident in HBM before the timed region.

Prints ONE JSON line: weight-elements/s over the whole job, the matrix-core roofline of the
dominant (fused transform) kernel measured with HIP events on the launch stream inside the
timed region, and the CPU oracle timed on the host cores on a bounded sample.

The loss pass of the fused kernel (forward transform, quantizer, inverse transform of the
rounding error, loss partials) runs its two contractions on the bfloat16 matrix pipe with every
float32 operand split exactly into three bfloat16 parts (6 + 3 part products, float32
accumulation); the gradient through the transformed weights is a second, shorter pass over the
same weights.  The roofline line prices the ALGORITHMIC work of the loss pass, 2 * 2k flop per
weight element, against the dense bfloat16 peak; the executed part products (4.5x as many
flops) and the float32 matrix peak the split replaces are given beside it for context.
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

BF16_MFMA_PEAK_TFLOPS = 2500.0
FP32_MFMA_PEAK_TFLOPS = 157.3
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the fused kernel on this workload, from the two rocprofv3 --pmc runs
# summarised in profiles/xform_core_c3_pair.md (FETCH_SIZE and WRITE_SIZE, each scaled by
# what the same counter reads for a plain 1 GiB copy); None for any other workload.
MEASURED_TRAFFIC_BYTES = {"c3_pair_3584x14336_k128_g128_b3": (2.0 * 168382 + 24288) * 1024}


def cpu_baseline(cfg, blocks, reps):
    """The oracle as it stands, on the first `blocks` transform blocks of the pair."""
    import numpy as np
    from oracle import cafeq_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
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
    return {"value": elems * reps / dt, "unit": "weight-elements/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d of %d transform blocks of the same pair (%.1f M weights), %d x (block inverse + "
                      "fwd+bwd), %.1f s" % (blocks, cfg["T"].shape[0], elems / 1e6, reps, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-blocks", type=int, default=112)
    ap.add_argument("--cpu-reps", type=int, default=4)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (the path is sharded by transform block "
                 "in design only); --gpus %d is not available" % args.gpus)

    import torch
    from paper_2511_19705_amd import cafeq, workloads as WL

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = WL.config3()
    k, g, bits, rep = cfg["k"], cfg["group"], cfg["bits"][0], cfg["rep"]
    A = torch.from_numpy(cfg["A"]).to(dev)
    B = torch.from_numpy(cfg["B"]).to(dev)
    T = torch.from_numpy(cfg["T"]).to(dev)
    elems = A.numel() + B.numel()

    def step():
        P, _ = cafeq.block_inverse(T)
        return cafeq.dual_proxy_loss_fwd_bwd(A, B, T, P, bits, g, rep, 5.0, want_grad=True)

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    cafeq.profile_enable(True)
    cafeq.profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_launch, core_ms = cafeq.profile_read()
    cafeq.profile_enable(False)
    losses = out[0].cpu().numpy()

    ms_per_step = dt / args.steps * 1e3
    value = elems * args.steps / dt
    # dominant kernel: the loss pass of the fused transform core, launched once per member.
    # Algorithmic work per launch: forward and inverse transform of its member, 2k flop per
    # element each; it reads every weight once (4 B per element).
    member = elems / 2.0
    flops_per_launch = 2.0 * 2.0 * k * member
    avg_launch_s = core_ms / 1e3 / max(n_launch, 1)
    achieved = flops_per_launch / avg_launch_s / 1e12
    executed = 9.0 * 2.0 * k * member / avg_launch_s / 1e12
    result = {
        "metric": "proxy-loss fwd+bwd weight-elements/s (9B-shaped MLP pair, dual transform)",
        "value": value, "unit": "weight-elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "rows_cols": [list(cfg["A"].shape), list(cfg["B"].shape)],
                   "block": k, "group": g, "bits": bits, "evals_per_s": args.steps / dt,
                   "step": "block inverse + dual proxy-loss fwd+bwd (loss pass + gradient pass per member)",
                   "contraction": "float32 operands split exactly into 3 bfloat16 parts, float32 accumulate",
                   "relative_l2_A": float((losses[2] / float((cfg["A"].astype("float64") ** 2).sum())) ** 0.5)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg["name"]),
                     "kernel": "xform_core_kernel<128,128,*,false> (loss pass)", "launches": n_launch,
                     "avg_launch_us": avg_launch_s * 1e6,
                     "algorithmic_flop_per_element": 4 * k, "algorithmic_bytes_per_element": 4,
                     "executed_part_product_tflops": executed,
                     "executed_frac_of_bf16_peak": executed / BF16_MFMA_PEAK_TFLOPS,
                     "achieved_over_fp32_mfma_peak": achieved / FP32_MFMA_PEAK_TFLOPS,
                     "hbm_frac_at_algorithmic_bytes": 4.0 * member / avg_launch_s / 1e9 / HBM_PEAK_GBS},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args.cpu_blocks, args.cpu_reps)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
