#!/usr/bin/env python3
"""The paper's SKLinear runtime grid (Sec. 4.1, Fig. 1) on one MI355X: square
layers of 8192 features, l in {1, 2, 3}, k in {16 .. 512}, against the dense
layer (torch.matmul, i.e. hipBLASLt) at the same shape.

    python -m paper_2601_15473_amd.grid_bench [--steps 50] [--tokens 4096]

Prints a markdown table: forward and forward+backward time of the sketched layer
(libsk) and of the dense layer, and their ratio.  Configurations the paper's size
rule excludes (2 l k (in + out) > in out) are marked as skipped, not run.  Inputs
are synthetic (workloads.generate); the paper states no batch size, so the token
count is a free parameter here.
"""
from __future__ import annotations

import argparse
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--tokens", type=int, default=0)
    args = ap.parse_args()

    import torch
    from . import libsk as sk
    from . import workloads as W
    from .device import DeviceLayer

    if not torch.cuda.is_available():
        sys.exit("grid_bench: no GPU visible")
    stream = torch.cuda.Stream()

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for _ in range(3):
                fn()
            e0.record(stream)
            for _ in range(n):
                fn()
            e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    f = W.PAPER_GRID_FEATURES
    T = args.tokens or W.PAPER_GRID_TOKENS
    x = torch.randn(T, f, device="cuda", dtype=torch.bfloat16)
    dY = torch.randn(T, f, device="cuda", dtype=torch.bfloat16)
    Wd = torch.randn(f, f, device="cuda", dtype=torch.bfloat16)
    dense_fwd = timed(lambda: torch.matmul(x, Wd.t()), args.steps)
    dense_all = timed(lambda: (torch.matmul(x, Wd.t()), torch.matmul(dY, Wd), torch.matmul(dY.t(), x)),
                      args.steps)
    print(f"dense {f}x{f}, {T} tokens, bf16: forward {dense_fwd:.4f} ms, forward+backward {dense_all:.4f} ms\n")
    print("| l | k | sketched fwd ms | fwd+bwd ms | fwd speed-up vs dense | fwd+bwd speed-up | TFLOP/s (fwd+bwd) |")
    print("|---|---|---|---|---|---|---|")
    for w in W.PAPER_GRID:
        if args.tokens:
            w = W.scaled(w, tokens=args.tokens)
        if 2 * w.l * w.k * (w.d_in + w.d_out) > w.d_in * w.d_out:   # the paper's size rule
            print(f"| {w.l} | {w.k} | skipped (no smaller than the dense layer) | | | | |")
            continue
        d = DeviceLayer(W.generate(w), sk, poison=False)

        def check(st):
            if st != sk.SK_OK:
                raise sk.SkError(st)
        fwd = timed(lambda: check(d.fwd(stream)), args.steps)
        both = timed(lambda: (check(d.fwd(stream)), check(d.bwd_input(stream)), check(d.bwd_weight(stream))),
                     args.steps)
        flops = 6.0 * w.tokens * w.R * (w.d_in + w.d_out)
        print(f"| {w.l} | {w.k} | {fwd:.4f} | {both:.4f} | {dense_fwd / fwd:.2f}x | {dense_all / both:.2f}x "
              f"| {flops / both / 1e9:.0f} |", flush=True)
        del d
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
