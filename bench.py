#!/usr/bin/env python3
"""Benchmark of the SKLinear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = forward + input gradient + factor/bias gradient (the three libsk
entry points) over one batch of synthetic input that is already resident in
HBM.  Prints ONE JSON line.  `value` is tokens per second of the whole step;
TFLOP/s and the per-call times ride along.  The roofline object is for the
dominant call of the step (the entry point that takes the most time), timed
live with HIP events on the launch stream: K back-to-back launches between
two events.  Buffers are rotated through enough copies to exceed the 256 MB
Infinity Cache ("cold"); the same loop on one buffer set is reported as warm.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

# HBM bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs of
# this script with --calibrate-copy), summed over the call's kernels and scaled by the
# same counters' reading for the 256 MiB calibration copy (FETCH_SIZE reads half the
# copied bytes on this machine, factor 2.0; WRITE_SIZE reads them exactly, factor 1.0).
# Source: profiles/c1_bert_base_ffn_up_hbm_traffic.txt.  Automatic plan only.
MEASURED_TRAFFIC_BYTES = {
    ("c1_bert_base_ffn_up", "fwd"): 39.6e6,
    ("c1_bert_base_ffn_up", "bwd_input"): 51.6e6,
    ("c1_bert_base_ffn_up", "bwd_weight"): 54.2e6,
}
# Kernels behind each entry point in the automatic plan for narrow sketches (R <= 128).
CALL_KERNELS = {
    "fwd": ["chain_small_kernel (fused)"],
    "bwd_input": ["gemm_bf16_kernel (split-K, NT)", "chain_small_kernel (expand)"],
    "bwd_weight": ["gemm_bf16_kernel (Z^T)", "gemm_bf16_kernel (split-K, column sums)",
                   "reduce_splits_kernel"],
    "bwd": ["dual_gemm_kernel (dY.U^T split-K beside Z^T)", "gemm_bf16_kernel (split-K, column sums)",
            "chain_small_kernel (expand, carrying the sum of the splits)"],
    "bwd_weight_first": ["gemm_bf16_kernel (dY.U^T)", "gemm_bf16_kernel (split-K, x^T.G)",
                         "reduce_splits_kernel"],
}

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
MFMA_F32_PEAK_TFLOPS = 157.3
INFINITY_CACHE_BYTES = 256 << 20


def algorithmic(w, op):
    """(flops, HBM bytes) one call must do: operands read once, results written
    once; the R-wide intermediate, its recomputation across tiles and cache
    re-reads are not counted."""
    e = 2 if w.dtype == "bf16" else 4
    T, i, o, R = w.tokens, w.d_in, w.d_out, w.R
    flops = 2 * T * R * (i + o)
    if op == "fwd":
        b = e * (T * (i + o) + R * (i + o) + o)
    elif op == "bwd_input":
        b = e * (T * (i + o) + R * (i + o))
    elif op == "bwd_weight":
        b = e * (T * (i + o) + i * R) + 4 * (R * o + o)
    elif op == "bwd":  # both gradients: x and dY in once, dX, dU, db out
        flops = 4 * T * R * (i + o)
        b = e * (T * (2 * i + o) + R * (i + o)) + 4 * (R * o + o)
    else:  # bwd_weight_first: x, dY and the fixed half of the second stage in, dA out
        h = R // 2
        flops = 2 * T * h * (i + o)
        b = e * (T * (i + o) + h * o) + 4 * i * h
    return flops, b


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c1_bert_base_ffn_up")
    ap.add_argument("--plan", type=int, default=0, help="0 auto, 1 fused, 2 two-pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-context", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--tokens", type=int, default=0, help="override the workload's token count")
    ap.add_argument("--single-call-backward", action="store_true",
                    help="one step = sk_linear_fwd + sk_linear_bwd (both gradients in one call)")
    ap.add_argument("--two-sided", action="store_true",
                    help="the two-sided reading of the layer: half of the workload's terms on each "
                         "side (same stage-matrix shapes), four calls per step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 256 MiB device-to-device copy (for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1")

    import torch
    from paper_2601_15473_amd import libsk as sk
    from paper_2601_15473_amd import workloads as W
    from paper_2601_15473_amd.device import DeviceLayer, TwoSidedDeviceLayer

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    w = W.BY_NAME[args.workload]
    if args.tokens:
        w = W.scaled(w, tokens=args.tokens)
    sk.sk_set_plan(args.plan)
    if args.two_sided:
        if w.l % 2:
            sys.exit("bench.py: --two-sided needs an even number of terms to split over the two sides")
        tensors = W.generate_two_sided(W.scaled(w, l=w.l // 2))
        DeviceLayer = TwoSidedDeviceLayer
    else:
        tensors = W.generate(w)

    # Buffer sets: enough copies that a full rotation exceeds twice the Infinity Cache.
    one = DeviceLayer(tensors, sk, poison=False)
    per_set = sum(t.numel() * t.element_size() for t in
                  (one.x, one.dY, one.y, one.dX, one.dU, one.db, one.ws, one.S_cat, one.U_cat))
    n_sets = max(2, min(64, int(np.ceil(2 * INFINITY_CACHE_BYTES / per_set))))
    sets = [one] + [DeviceLayer(tensors, sk, poison=False) for _ in range(n_sets - 1)]

    stream = torch.cuda.Stream()
    ops = ("fwd", "bwd_input", "bwd_weight") + (("bwd_weight_first",) if args.two_sided else ())
    if args.single_call_backward:
        if args.two_sided:
            sys.exit("bench.py: --single-call-backward and --two-sided do not combine")
        ops = ("fwd", "bwd")

    def call(d, op):
        st = getattr(d, op)(stream)
        if st != sk.SK_OK:
            raise sk.SkError(st)

    def step(d):
        for op in ops:
            call(d, op)

    def timed(fn, n):
        """ms per iteration of fn(i), n iterations between two events on the launch stream."""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            e0.record(stream)
            for i in range(n):
                fn(i)
            e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            step(sets[i % n_sets])
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps, cold (rotating buffer sets) ----
    t0 = time.perf_counter()
    ms_step = timed(lambda i: step(sets[i % n_sets]), args.steps)
    wall = time.perf_counter() - t0
    ms_step_warm = timed(lambda i: step(one), args.steps)

    # ---- the same step with both gradients from one call (sk_linear_bwd), same protocol ----
    ms_step_single = None
    if not args.two_sided and not args.single_call_backward:
        def step_single(d):
            call(d, "fwd")
            call(d, "bwd")
        with torch.cuda.stream(stream):
            for i in range(args.warmup):
                step_single(sets[i % n_sets])
        ms_step_single = timed(lambda i: step_single(sets[i % n_sets]), args.steps)

    # ---- per-call times, same protocol ----
    per_op = {}
    for op in ops:
        per_op[op] = {
            "ms": timed(lambda i, op=op: call(sets[i % n_sets], op), args.steps),
            "ms_warm": timed(lambda i, op=op: call(one, op), args.steps),
        }
    flops_step = bytes_step = 0
    for op in ops:
        f, b = algorithmic(w, op)
        flops_step += f
        bytes_step += b
        per_op[op].update(tflops=f / per_op[op]["ms"] / 1e9, gbs=b / per_op[op]["ms"] / 1e6)

    # which roofline binds: arithmetic intensity against the ridge point
    peak_tf = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    t_mfma = flops_step / (peak_tf * 1e12)
    t_hbm = bytes_step / (HBM_PEAK_GBS * 1e9)
    bound = "mfma" if t_mfma > t_hbm else "hbm"
    dom = max(ops, key=lambda o: per_op[o]["ms"])
    f_dom, b_dom = algorithmic(w, dom)
    if bound == "hbm":
        achieved, peak, unit = b_dom / per_op[dom]["ms"] / 1e6, HBM_PEAK_GBS, "GB/s"
    else:
        achieved, peak, unit = f_dom / per_op[dom]["ms"] / 1e9, peak_tf, "TFLOP/s"
    traffic = (MEASURED_TRAFFIC_BYTES.get((w.name, dom))
               if args.plan == 0 and not args.tokens and not args.two_sided else None)  # none measured for 'bwd'
    roofline = {
        "bound": bound, "kernel": f"sk_linear_{dom}", "launch": "one call of the entry point",
        "kernels_in_call": CALL_KERNELS[dom] if w.R <= 128 and w.dtype == "bf16" else None,
        "achieved": achieved, "peak": peak,
        "unit": unit, "frac": achieved / peak, "traffic": traffic,
        "step_frac": max(t_mfma, t_hbm) / (ms_step * 1e-3),
        "algorithmic_bytes": b_dom, "algorithmic_flops": f_dom, "ms": per_op[dom]["ms"],
    }

    out = {
        "metric": "SKLinear fwd+bwd tokens/s (TFLOP/s and roofline fraction alongside)",
        "value": w.tokens / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + (" (two-sided: %d + %d terms)" % (w.l // 2, w.l // 2) if args.two_sided else ""),
                   "tokens": w.tokens, "in": w.d_in, "out": w.d_out,
                   "l": w.l, "k": w.k, "plan": args.plan, "buffer_sets": n_sets,
                   "calls_per_step": list(ops),
                   "cache": "cold (buffer sets rotate, total > 2x Infinity Cache)"},
        "tflops": flops_step / (ms_step * 1e-3) / 1e12,
        "ms_per_step_warm": ms_step_warm,
        "wall_s_timed_region": wall,
        "per_call": per_op,
        "roofline": roofline,
    }
    if ms_step_single is not None:
        out["single_call_backward"] = {
            "what": "the same step as sk_linear_fwd + sk_linear_bwd (both gradients in one call, "
                    "kernels of the two gradients sharing launches); not used for `value`",
            "ms_per_step": ms_step_single, "tokens_per_s": w.tokens / (ms_step_single * 1e-3)}

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibrate_copy_bytes"] = 256 << 20

    if not args.no_dense_context:
        # the dense layer the sketch replaces (hipBLASLt through torch.matmul): context only
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        Wd = torch.randn(w.d_out, w.d_in, device="cuda", dtype=dt)
        x, dY = one.x, one.dY

        def dense(i):
            torch.matmul(x, Wd.t())
            torch.matmul(dY, Wd)
            torch.matmul(dY.t(), x)
        with torch.cuda.stream(stream):
            for i in range(5):
                dense(i)
        ms_dense = timed(dense, max(10, args.steps // 4))
        out["dense_context"] = {"ms_per_step": ms_dense, "kind": "torch.matmul (hipBLASLt) x3",
                                "tflops": 6 * w.tokens * w.d_in * w.d_out / ms_dense / 1e9}

    if not args.no_cpu_baseline:
        from oracle import sklinear as O
        v = {n: a.astype(np.float64) for n, a in tensors.value.items()}

        if args.two_sided:
            from oracle import sklinear_two_sided as O2
            terms = (v["S1"], v["U1"], v["U2"], v["S2"])

            def oracle_step():
                O2.forward(v["x"], *terms, v["b"])
                O2.grad_input(v["dY"], *terms)
                O2.grad_second_stage(v["x"], v["S1"], v["dY"])
                O2.grad_first_stage(v["x"], v["S2"], v["dY"])
                O2.grad_bias(v["dY"])
        else:
            def oracle_step():
                O.forward(v["x"], v["S"], v["U"], v.get("b"))
                O.grad_input(v["dY"], v["S"], v["U"])
                O.grad_factors(v["x"], v["S"], v["dY"])
                O.grad_bias(v["dY"])
        oracle_step()
        reps, t_begin = 0, time.perf_counter()
        while True:
            oracle_step()
            reps += 1
            el = time.perf_counter() - t_begin
            if el >= args.cpu_seconds or (reps >= 3 and el >= 0.5 * args.cpu_seconds):
                break
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        out["cpu_baseline"] = {
            "value": w.tokens * reps / el, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} full passes of {w.name} (fwd + both gradients, fp64 numpy/OpenBLAS)",
        }

    print(json.dumps(out))


if __name__ == "__main__":
    main()
