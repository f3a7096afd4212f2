#!/usr/bin/env python3
"""Per-call time and fraction of the roofline over a matrix of layer shapes, sketch widths
and token counts (bf16, random data, a few rotating input sets): a check that the
automatic plans hold up away from the benchmark configurations.

    python -m paper_2601_15473_amd.shape_sweep                     # the built-in matrix
    python -m paper_2601_15473_amd.shape_sweep T,in,out,R [...]    # given cases, every plan

The roofline of a call is the larger of its algorithmic HBM time at 8 TB/s (inputs read
once, outputs written once) and its MFMA time at 2.5 PFLOP/s.
"""
from __future__ import annotations

import sys


def main():
    import torch
    from . import libsk as sk

    if not torch.cuda.is_available():
        sys.exit("shape_sweep: no GPU visible")
    stream = torch.cuda.Stream()

    def run(T, i, o, R):
        l, k = 1, R
        dt = sk.DTYPES["bf16"]
        nset = max(2, min(8, int(600e6 // (2 * T * (i + o)) + 1)))

        def mk(*shape):
            return torch.randn(*shape, device="cuda", dtype=torch.float32).to(torch.bfloat16)

        S, U, b = mk(i, R) * R ** -0.5, mk(R, o) * R ** -0.5, mk(o)
        xs = [mk(T, i) for _ in range(nset)]
        dYs = [mk(T, o) for _ in range(nset)]
        y = torch.empty(T, o, device="cuda", dtype=torch.bfloat16)
        dX = torch.empty(T, i, device="cuda", dtype=torch.bfloat16)
        dU = torch.empty(R, o, device="cuda")
        db = torch.empty(o, device="cuda")
        args = (T, i, o, l, k, dt)
        need = max(sk.sk_linear_workspace_bytes(op, *args) for op in (0, 1, 2))
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        calls = {
            "fwd": lambda n: sk.sk_linear_fwd(xs[n], S, U, b, y, *args, ws, need, stream),
            "bwd_input": lambda n: sk.sk_linear_bwd_input(dYs[n], S, U, dX, *args, ws, need, stream),
            "bwd_weight": lambda n: sk.sk_linear_bwd_weight(xs[n], S, dYs[n], dU, db, *args, ws, need, stream),
        }
        flops = 2 * T * R * (i + o)
        byts = {"fwd": 2 * T * (i + o), "bwd_input": 2 * T * (i + o), "bwd_weight": 2 * T * (i + o) + 4 * R * o}
        out = []
        for op, fn in calls.items():
            reps = 20 if T * (i + o) < 3e8 else 6
            with torch.cuda.stream(stream):
                for n in range(2):
                    sk.check(fn(n % nset))
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for n in range(reps):
                    fn(n % nset)
                e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / reps * 1e3
            ideal = max(byts[op] / 8e12, flops / 2.5e15) * 1e6
            out.append((op, us, ideal / us))
        print(f"T={T:6d} {i:5d}->{o:5d} R={R:4d} | " +
              "  ".join(f"{op} {us:8.1f}us {fr:.2f}" for op, us, fr in out), flush=True)

    if len(sys.argv) > 1:
        cases = [tuple(map(int, c.split(","))) for c in sys.argv[1:]]
        for plan, name in ((0, "automatic"), (1, "fused"), (3, "split + expand"), (2, "two GEMMs")):
            sk.sk_set_plan(plan)
            print("plan:", name)
            for case in cases:
                run(*case)
        sk.sk_set_plan(0)
        return
    layers = [(768, 3072), (3072, 768), (1024, 4096), (4096, 1024), (2048, 2048), (4096, 11008), (8192, 8192)]
    for (i, o) in layers:
        for R in (32, 128, 512, 2048):
            if R > min(i, o):
                continue
            for T in (1024, 4096, 16384, 65536):
                if T * (i + o) * 2 > 3.2e9:
                    continue
                run(T, i, o, R)


if __name__ == "__main__":
    main()
