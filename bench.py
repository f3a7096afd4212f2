#!/usr/bin/env python3
"""Benchmark of the SKLinear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = forward (sk_linear_fwd) + input, factor and bias gradients
(sk_linear_bwd, both gradients in one call) over one batch of synthetic input
that is already resident in HBM.  Prints ONE JSON line.  The same step through
the three separate entry points is timed beside it (`three_call_step`), and
every entry point by itself (`per_call`).

Headline (`value`, `config`, `roofline`, `cpu_baseline`): the largest benchmark
configuration, c4_llm_mlp, unless --workload names another.  `value` is tokens
per second of the whole step: after W warm-up steps, five batches of exactly K
steps each are timed between two HIP events on the launch stream and the median
batch is reported (all five are listed).  Buffer sets rotate so that a full
rotation exceeds twice the 256 MB Infinity Cache ("cold"); the same loop on one
buffer set is reported as warm.

`roofline` is for the dominant KERNEL of the step, named as a profiler prints
it: the same K steps run once more with a pair of events around every kernel
(include/sk_debug.h), and achieved = the flops (or bytes) the kernel's launches
must do / the time between their events.  `traffic` is the HBM bytes per launch
that rocprofv3's FETCH_SIZE / WRITE_SIZE counters measured for that kernel, read
from the summary under profiles/ (null when there is none for this workload).
`measured_peak` holds what this GPU gives a plain device copy and a large square
bf16 GEMM through hipBLASLt, and the fractions against those.

`configs` carries every other benchmark configuration (c1, each rank of c2,
c3 up and down) timed by the same protocol with 200 steps per batch, with
per-call times, the fraction of the binding roofline and the dense layer the
sketch replaces beside each; c0 (fp32, launch-bound) rides along as a parity
stamp against the oracle, not as a timing.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
MFMA_F32_PEAK_TFLOPS = 157.3
INFINITY_CACHE_BYTES = 256 << 20
BATCHES = 5


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
    elif op == "bwd":
        # both gradients from one call: counted as the two gradient calls it stands for (dY read by
        # each, as the library does); a single pass over dY would need e * T * out bytes fewer
        flops = 4 * T * R * (i + o)
        b = e * (T * (i + o) + R * (i + o)) + e * (T * (i + o) + i * R) + 4 * (R * o + o)
    else:  # bwd_weight_first: x, dY and the fixed half of the second stage in, dA out
        h = R // 2
        flops = 2 * T * h * (i + o)
        b = e * (T * (i + o) + h * o) + 4 * i * h
    return flops, b


def measured_traffic(workload_name):
    """{(kernel name, work-groups): HBM bytes per launch} from the rocprofv3 counter summary
    of this workload under profiles/ (lines `TRAFFIC <tab> kernel <tab> groups <tab> fetch
    bytes <tab> write bytes`, already scaled by the copy calibration stated in the file)."""
    path = os.path.join(ROOT, "profiles", f"{workload_name}_hbm_traffic.txt")
    out = {}
    if not os.path.exists(path):
        return out, None
    for line in open(path):
        f = line.rstrip("\n").split("\t")
        if len(f) == 5 and f[0] == "TRAFFIC":
            out[(f[1].strip(), int(f[2]))] = float(f[3]) + float(f[4])
    return out, os.path.relpath(path, ROOT)


class Harness:
    def __init__(self, torch, sk, W, device_mod, args):
        self.torch, self.sk, self.W, self.dm, self.args = torch, sk, W, device_mod, args
        self.stream = torch.cuda.Stream()

    def timed(self, fn, n):
        """ms per iteration of fn(i): n iterations between two events on the launch stream."""
        torch = self.torch
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            e0.record(self.stream)
            for i in range(n):
                fn(i)
            e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def batches(self, fn, n):
        """Five batches of n iterations: (median ms per iteration, all five)."""
        ms = [self.timed(fn, n) for _ in range(BATCHES)]
        return statistics.median(ms), ms

    def call(self, d, op):
        st = getattr(d, op)(self.stream)
        if st != self.sk.SK_OK:
            raise self.sk.SkError(st)

    def kernel_times(self, step, sets, steps):
        """The step run `steps` times with events around every kernel: per kernel (name,
        work-groups), launches per step, mean ms per launch, flops and bytes per launch."""
        sk, torch = self.sk, self.torch
        cap = 24 * steps
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            sk.sk_profile_begin(cap)
            try:
                for i in range(steps):
                    step(sets[i % len(sets)])
            finally:
                recs = sk.sk_profile_end(cap)
        torch.cuda.synchronize()
        agg = {}
        for name, ms, groups, flops, nbytes in recs:
            a = agg.setdefault((name, groups), dict(kernel=name, groups=groups, launches=0, ms=0.0, flops=0.0, bytes=0.0))
            a["launches"] += 1
            a["ms"] += ms
            a["flops"] += flops
            a["bytes"] += nbytes
        out = []
        for a in agg.values():
            n = a["launches"]
            out.append(dict(kernel=a["kernel"], groups=a["groups"], launches_per_step=n / steps,
                            ms_per_launch=a["ms"] / n, ms_per_step=a["ms"] / steps,
                            flops_per_launch=a["flops"] / n, bytes_per_launch=a["bytes"] / n))
        out.sort(key=lambda k: -k["ms_per_step"])
        return out

    def dense(self, w, x, dY, n):
        """The dense layer the sketch replaces (hipBLASLt through torch.matmul): context only."""
        torch = self.torch
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        Wd = torch.randn(w.d_out, w.d_in, device="cuda", dtype=dt)

        def step(i):
            torch.matmul(x, Wd.t())
            torch.matmul(dY, Wd)
            torch.matmul(dY.t(), x)
        with torch.cuda.stream(self.stream):
            for i in range(3):
                step(i)
        ms, _ = self.batches(step, n)
        return ms

    def measure(self, w, steps, warmup, headline):
        """One workload by the protocol of the module docstring."""
        torch, sk, W, args = self.torch, self.sk, self.W, self.args
        if args.two_sided and headline:
            tensors = W.generate_two_sided(W.scaled(w, l=w.l // 2))
            Layer = self.dm.TwoSidedDeviceLayer
        else:
            tensors = W.generate(w)
            Layer = self.dm.DeviceLayer
        one = Layer(tensors, sk, poison=False)
        per_set = sum(t.numel() * t.element_size() for t in
                      (one.x, one.dY, one.y, one.dX, one.dU, one.db, one.ws, one.S_cat, one.U_cat))
        n_sets = max(2, min(64, int(np.ceil(2 * INFINITY_CACHE_BYTES / per_set))))
        sets = [one] + [Layer(tensors, sk, poison=False) for _ in range(n_sets - 1)]

        # the step: forward, then both gradients from sk_linear_bwd (one call whose kernels share
        # launches where that pays); --three-calls times the three separate entry points instead
        ops = ("fwd", "bwd")
        if args.three_calls:
            ops = ("fwd", "bwd_input", "bwd_weight")
        if args.two_sided and headline:
            ops = ("fwd", "bwd_input", "bwd_weight", "bwd_weight_first")

        def step(d):
            for op in ops:
                self.call(d, op)

        with torch.cuda.stream(self.stream):
            for i in range(warmup):
                step(sets[i % n_sets])
        torch.cuda.synchronize()

        t0 = time.perf_counter()
        ms_step, ms_batches = self.batches(lambda i: step(sets[i % n_sets]), steps)
        wall = time.perf_counter() - t0
        ms_warm = self.timed(lambda i: step(one), steps)

        res = {"ms_per_step": ms_step, "ms_per_step_batches": ms_batches, "ms_per_step_warm": ms_warm,
               "tokens": w.tokens, "in": w.d_in, "out": w.d_out, "l": w.l, "k": w.k, "R": w.R, "dtype": w.dtype,
               "steps_per_batch": steps, "buffer_sets": n_sets, "wall_s_timed_region": wall}

        if ops == ("fwd", "bwd"):
            def step_three(d):
                for op in ("fwd", "bwd_input", "bwd_weight"):
                    self.call(d, op)
            with torch.cuda.stream(self.stream):
                for i in range(min(warmup, 5)):
                    step_three(sets[i % n_sets])
            ms_three, _ = self.batches(lambda i: step_three(sets[i % n_sets]), steps)
            res["three_call_ms_per_step"] = ms_three

        per_op, flops_step, bytes_step = {}, 0, 0
        timed_ops = ops if (args.two_sided and headline) else ("fwd", "bwd", "bwd_input", "bwd_weight")
        for op in timed_ops:
            ms, _ = self.batches(lambda i, op=op: self.call(sets[i % n_sets], op), steps)
            f, b = algorithmic(w, op)
            if op in ops:
                flops_step += f
                bytes_step += b
            per_op[op] = {"ms": ms, "tflops": f / ms / 1e9, "gbs": b / ms / 1e6}
        peak_tf = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
        t_mfma = flops_step / (peak_tf * 1e12)
        t_hbm = bytes_step / (HBM_PEAK_GBS * 1e9)
        res.update(per_call=per_op, bound="mfma" if t_mfma > t_hbm else "hbm",
                   step_frac=max(t_mfma, t_hbm) / (ms_step * 1e-3),
                   tflops=flops_step / (ms_step * 1e-3) / 1e12, gbs=bytes_step / (ms_step * 1e-3) / 1e9,
                   tokens_per_s=w.tokens / (ms_step * 1e-3),
                   algorithmic_flops_per_step=flops_step, algorithmic_bytes_per_step=bytes_step)
        for op in timed_ops:
            f, b = algorithmic(w, op)
            per_op[op]["frac"] = max(f / (peak_tf * 1e12), b / (HBM_PEAK_GBS * 1e9)) / (per_op[op]["ms"] * 1e-3)

        res["kernels"] = self.kernel_times(step, sets, min(steps, 10))
        if not args.no_dense_context:
            ms_dense = self.dense(w, one.x, one.dY, max(5, steps // 4))
            res["dense_context"] = {
                "ms_per_step": ms_dense, "kind": "torch.matmul (hipBLASLt) x3: the dense layer's forward and two gradients",
                "tflops": 6 * w.tokens * w.d_in * w.d_out / ms_dense / 1e9,
                "sketched_over_dense_time": ms_step / ms_dense,
                "sketched_over_dense_flops": flops_step / (6 * w.tokens * w.d_in * w.d_out)}
        del sets, one
        torch.cuda.empty_cache()
        return res, tensors, ops


def measured_peaks(torch, stream, sk):
    """What this GPU gives a plain device-to-device copy (bytes read + written per second)
    and a large square bf16 GEMM through hipBLASLt -- and, like for like, what this library's
    own GEMM kernel reaches on the same 8192^3 product (the two GEMMs of sk_linear_fwd on a
    layer with tokens = in = out = R = 8192)."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best_copy = 0.0
    with torch.cuda.stream(stream):
        for _ in range(2):
            dst.copy_(src)
        for _ in range(3):
            e0.record(stream)
            for _ in range(5):
                dst.copy_(src)
            e1.record(stream)
            e1.synchronize()
            best_copy = max(best_copy, 2.0 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    m = 8192
    a = torch.randn(m, m, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(m, m, device="cuda", dtype=torch.bfloat16)
    best_gemm = 0.0
    with torch.cuda.stream(stream):
        for _ in range(3):
            torch.matmul(a, b)
        for _ in range(3):
            e0.record(stream)
            for _ in range(10):
                torch.matmul(a, b)
            e1.record(stream)
            e1.synchronize()
            best_gemm = max(best_gemm, 2.0 * m ** 3 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    del a, b
    own = 0.0
    x = torch.randn(m, m, device="cuda", dtype=torch.bfloat16)
    S = torch.randn(m, m, device="cuda", dtype=torch.bfloat16) * 0.01
    U = torch.randn(m, m, device="cuda", dtype=torch.bfloat16) * 0.01
    y = torch.empty(m, m, device="cuda", dtype=torch.bfloat16)
    args = (m, m, m, 1, m, sk.SK_BF16)
    ws_bytes = sk.sk_linear_workspace_bytes(sk.SK_OP_FWD, *args)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    with torch.cuda.stream(stream):
        for _ in range(2):
            sk.check(sk.sk_linear_fwd(x, S, U, None, y, *args, ws, ws_bytes, stream))
        for _ in range(3):
            e0.record(stream)
            for _ in range(5):
                sk.check(sk.sk_linear_fwd(x, S, U, None, y, *args, ws, ws_bytes, stream))
            e1.record(stream)
            e1.synchronize()
            own = max(own, 2 * 2.0 * m ** 3 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    del x, S, U, y, ws
    torch.cuda.empty_cache()
    return {"hbm_copy_gbs": best_copy, "hbm_copy_what": "1 GiB device-to-device copy, bytes read + written per second",
            "mfma_bf16_tflops": best_gemm, "mfma_what": "8192^3 bf16 GEMM, torch.matmul (hipBLASLt)",
            "own_gemm_bf16_tflops": own,
            "own_gemm_what": "the same 8192^3 product by this library's GEMM kernel (sk_linear_fwd with "
                             "tokens = in = out = R = 8192: two such GEMMs per call)"}


def parity_stamp(torch, sk, W, dm):
    """Config 0 (tiny, fp32) through the three calls against the oracle: max relative error."""
    from oracle import sklinear as O
    w = W.TINY
    t = W.generate(w)
    dev = dm.DeviceLayer(t, sk)
    dev.run_all()
    v = {n: a.astype(np.float64) for n, a in t.value.items()}
    want = {"y": O.forward(v["x"], v["S"], v["U"], v["b"]), "dX": O.grad_input(v["dY"], v["S"], v["U"]),
            "dU": O.grad_factors(v["x"], v["S"], v["dY"]).reshape(w.R, w.d_out), "db": O.grad_bias(v["dY"])}
    worst = 0.0
    for n, ref in want.items():
        got = getattr(dev, n).detach().to(torch.float64).cpu().numpy()
        r2 = ref.reshape(ref.shape[0], -1) if ref.ndim > 1 else ref.reshape(1, -1)
        rms = np.sqrt(np.mean(r2 * r2, axis=1, keepdims=True))
        worst = max(worst, float(np.max(np.abs(got.reshape(r2.shape) - r2) / np.maximum(np.abs(r2), rms))))
    return {"workload": w.name, "max_rel_err_vs_oracle": worst, "tolerance": 1e-4, "ok": bool(worst <= 1e-4),
            "note": "fp32, launch-bound: a parity stamp, not a timing"}


def cpu_baseline(w, tensors, seconds, two_sided):
    """The oracle as it stands on the host cores, on a bounded sample of the headline
    workload: the first rows of the batch (all of it when that is quick), whole passes
    (forward + both gradients) repeated for about `seconds`."""
    from oracle import sklinear as O
    sample = min(w.tokens, 4096)
    v = {n: (a[:sample] if n in ("x", "dY") else a).astype(np.float64) for n, a in tensors.value.items()}
    if two_sided:
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
        if el >= seconds or (reps >= 3 and el >= 0.5 * seconds):
            break
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    return {"value": sample * reps / el, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{reps} passes over the first {sample} of {w.tokens} tokens of {w.name} "
                      f"(forward + both gradients, fp64 numpy/OpenBLAS, {el:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="steps per timed batch of the headline workload")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4_llm_mlp", help="the headline workload")
    ap.add_argument("--plan", type=int, default=0, help="0 auto, 1 fused, 2 two GEMMs, 3 split + expand")
    ap.add_argument("--no-configs", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-context", action="store_true")
    ap.add_argument("--no-measured-peak", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--tokens", type=int, default=0, help="override the headline workload's token count")
    ap.add_argument("--three-calls", action="store_true",
                    help="one step = sk_linear_fwd + sk_linear_bwd_input + sk_linear_bwd_weight instead of "
                         "sk_linear_fwd + sk_linear_bwd (both gradients in one call)")
    ap.add_argument("--two-sided", action="store_true",
                    help="the two-sided reading of the layer: half of the workload's terms on each "
                         "side (same stage-matrix shapes), four calls per step")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="force a plan parameter (sk_set_tuning), e.g. narrow_bwd=0; for sweeps")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1")

    import torch
    from paper_2601_15473_amd import device as dm
    from paper_2601_15473_amd import libsk as sk
    from paper_2601_15473_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.three_calls and args.two_sided:
        sys.exit("bench.py: --two-sided already times the separate calls (four per step)")
    w = W.BY_NAME[args.workload]
    if args.tokens:
        w = W.scaled(w, tokens=args.tokens)
    if args.two_sided and w.l % 2:
        sys.exit("bench.py: --two-sided needs an even number of terms to split over the two sides")
    sk.sk_set_plan(args.plan)
    for kv in args.tune:
        knob, _, value = kv.partition("=")
        sk.sk_set_tuning(getattr(sk, "SK_TUNE_" + knob.upper()), int(value))
    h = Harness(torch, sk, W, dm, args)

    head, tensors, ops = h.measure(w, args.steps, args.warmup, headline=True)

    # ---- roofline of the dominant kernel of the step ----
    dom = head["kernels"][0]
    intensity = dom["flops_per_launch"] / max(dom["bytes_per_launch"], 1.0)
    peak_tf = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    ridge = peak_tf * 1e12 / (HBM_PEAK_GBS * 1e9)
    traffic_table, traffic_src = measured_traffic(w.name) if args.plan == 0 and not args.tokens and \
        not args.two_sided else ({}, None)
    traffic = traffic_table.get((dom["kernel"], dom["groups"]))
    if intensity >= ridge:
        bound, unit, peak = "mfma", "TFLOP/s", peak_tf
        achieved = dom["flops_per_launch"] / (dom["ms_per_launch"] * 1e-3) / 1e12
    else:
        bound, unit, peak = "hbm", "GB/s", HBM_PEAK_GBS
        achieved = dom["bytes_per_launch"] / (dom["ms_per_launch"] * 1e-3) / 1e9
    roofline = {
        "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
        "traffic": traffic, "traffic_source": traffic_src if traffic is not None else None,
        "kernel": dom["kernel"], "work_groups": dom["groups"], "launches_per_step": dom["launches_per_step"],
        "ms_per_launch": dom["ms_per_launch"], "share_of_step": dom["ms_per_step"] / head["ms_per_step"],
        "algorithmic_flops_per_launch": dom["flops_per_launch"], "algorithmic_bytes_per_launch": dom["bytes_per_launch"],
        "how": "events around every kernel over %d steps (include/sk_debug.h); launches of one kernel averaged"
               % min(args.steps, 10),
        "step_frac": head["step_frac"], "step_bound": head["bound"],
    }

    out = {
        "metric": "SKLinear fwd+bwd tokens/s (TFLOP/s and roofline fraction alongside)",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + (" (two-sided: %d + %d terms)" % (w.l // 2, w.l // 2) if args.two_sided else ""),
                   "tokens": w.tokens, "in": w.d_in, "out": w.d_out,
                   "l": w.l, "k": w.k, "plan": args.plan, "buffer_sets": head["buffer_sets"],
                   "calls_per_step": list(ops),
                   "timing": "median of %d batches of %d steps" % (BATCHES, args.steps),
                   "cache": "cold (buffer sets rotate, total > 2x Infinity Cache)"},
        "tflops": head["tflops"],
        "ms_per_step_batches": head["ms_per_step_batches"],
        "ms_per_step_warm": head["ms_per_step_warm"],
        "wall_s_timed_region": head["wall_s_timed_region"],
        "per_call": head["per_call"],
        "roofline": roofline,
        "kernels": head["kernels"],
    }
    if "three_call_ms_per_step" in head:
        out["three_call_step"] = {
            "what": "the same step as sk_linear_fwd + sk_linear_bwd_input + sk_linear_bwd_weight (three entry points, "
                    "dY read by both gradient calls); not used for `value`",
            "ms_per_step": head["three_call_ms_per_step"],
            "tokens_per_s": w.tokens / (head["three_call_ms_per_step"] * 1e-3)}
    if "dense_context" in head:
        out["dense_context"] = head["dense_context"]

    mp = None
    if not args.no_measured_peak:
        mp = measured_peaks(torch, h.stream, sk)
        mp["roofline_frac_of_measured"] = achieved / (mp["mfma_bf16_tflops"] if bound == "mfma" else mp["hbm_copy_gbs"])
        t_m = head["algorithmic_flops_per_step"] / (mp["mfma_bf16_tflops"] * 1e12)
        t_h = head["algorithmic_bytes_per_step"] / (mp["hbm_copy_gbs"] * 1e9)
        mp["step_frac_of_measured"] = max(t_m, t_h) / (head["ms_per_step"] * 1e-3)
        out["measured_peak"] = mp

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibrate_copy_bytes"] = 256 << 20
        del src, dst

    if not args.no_configs:
        cfgs = {}
        for cw in (W.BERT_BASE_FFN_UP,) + W.BERT_BASE_PROJ + (W.BERT_LARGE_FFN_UP, W.BERT_LARGE_FFN_DOWN, W.LLM_MLP):
            if cw.name == w.name and not args.tokens and not args.two_sided:
                continue   # the headline itself
            big = cw.tokens * cw.R * (cw.d_in + cw.d_out) > 1e12
            r, _, _ = h.measure(cw, 20 if big else 200, 5 if big else 20, headline=False)
            r["kernels"] = r["kernels"][:6]
            r.pop("wall_s_timed_region")
            if mp is not None:
                t_m = r["algorithmic_flops_per_step"] / (mp["mfma_bf16_tflops"] * 1e12)
                t_h = r["algorithmic_bytes_per_step"] / (mp["hbm_copy_gbs"] * 1e9)
                r["step_frac_of_measured"] = max(t_m, t_h) / (r["ms_per_step"] * 1e-3)
            cfgs[cw.name] = r
        cfgs[W.TINY.name] = parity_stamp(torch, sk, W, dm)
        out["configs"] = cfgs

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, tensors, args.cpu_seconds, args.two_sided)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
