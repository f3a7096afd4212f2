"""Two-sided layer on the GPU against its fp64 oracle: forward, input gradient and
second-stage gradient through the one-sided entry points on the concatenated stage
matrices (2 l terms), first-stage gradient through sk_linear_bwd_weight_first."""
import numpy as np
import pytest
import torch

from oracle import sklinear_two_sided as O2
from paper_2601_15473_amd import workloads as W

pytestmark = pytest.mark.gpu

from skgpu import TOL, rel_err, to_dev, to_f64  # noqa: E402

CASES = [
    W.Workload("two_f32", 150, 96, 80, 2, 16, "f32", seed=21),
    W.Workload("two_bf16_small", 333, 208, 176, 1, 16, "bf16", seed=22),
    W.Workload("two_bf16_bert_base", 1000, 768, 3072, 1, 64, "bf16", seed=23),   # R' = 128 like c1
    W.Workload("two_bf16_square", 700, 768, 768, 2, 64, "bf16", seed=24),
    W.Workload("two_bf16_wide", 600, 1024, 4096, 2, 128, "bf16", seed=25),       # R' = 512 like c3
    # the benchmark's own shape: the first GEMM of the first-stage gradient (64 tiles over a
    # contraction 3072 long) runs split into fp32 slabs
    W.Workload("two_bf16_bert_base_full", 4096, 768, 3072, 1, 64, "bf16", seed=27),
    # long ragged contractions on both sides, ragged token tile
    W.Workload("two_bf16_long_ragged", 520, 4112, 2064, 1, 48, "bf16", seed=28),
    W.Workload("two_f32_long_ragged", 200, 1040, 2064, 1, 16, "f32", seed=29),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_two_sided_parity(w):
    from paper_2601_15473_amd import libsk as sk
    print(f"case {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l}+{w.l} k={w.k} {w.dtype}", flush=True)
    sk.sk_set_plan(0)
    t = W.generate_two_sided(w)
    l2, k, R = 2 * w.l, w.k, 2 * w.l * w.k
    half = w.l * w.k
    dt = sk.DTYPES[w.dtype]
    td = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    d = {n: to_dev(t.stored[n], w.dtype) for n in ("x", "dY", "b", "A_cat", "B_cat")}
    nan = float("nan")
    y = torch.full((w.tokens, w.d_out), nan, dtype=td, device="cuda")
    dX = torch.full((w.tokens, w.d_in), nan, dtype=td, device="cuda")
    dB = torch.full((R, w.d_out), nan, dtype=torch.float32, device="cuda")
    db = torch.full((w.d_out,), nan, dtype=torch.float32, device="cuda")
    dA = torch.full((w.d_in, half), nan, dtype=torch.float32, device="cuda")
    args = (w.tokens, w.d_in, w.d_out, l2, k, dt)
    need = max(sk.sk_linear_workspace_bytes(op, *args) for op in range(4))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    sk.check(sk.sk_linear_fwd(d["x"], d["A_cat"], d["B_cat"], d["b"], y, *args, ws, need))
    sk.check(sk.sk_linear_bwd_input(d["dY"], d["A_cat"], d["B_cat"], dX, *args, ws, need))
    sk.check(sk.sk_linear_bwd_weight(d["x"], d["A_cat"], d["dY"], dB, db, *args, ws, need))
    sk.check(sk.sk_linear_bwd_weight_first(d["x"], d["B_cat"], d["dY"], dA, w.tokens, w.d_in, w.d_out,
                                           l2, k, half, half, dt, ws, need))
    torch.cuda.synchronize()
    v = {n: a.astype(np.float64) for n, a in t.value.items()}
    terms = (v["S1"], v["U1"], v["U2"], v["S2"])
    want = dict(
        y=O2.forward(v["x"], *terms, v["b"]),
        dX=O2.grad_input(v["dY"], *terms),
        dU1=O2.grad_second_stage(v["x"], v["S1"], v["dY"]).reshape(half, w.d_out),
        # dA [in, l*k]: column i*k + j is the gradient of column j of U2_i
        dU2=np.transpose(O2.grad_first_stage(v["x"], v["S2"], v["dY"]), (1, 0, 2)).reshape(w.d_in, half),
        db=O2.grad_bias(v["dY"]),
    )
    got = dict(y=to_f64(y), dX=to_f64(dX), dU1=to_f64(dB[:half]), dU2=to_f64(dA), db=to_f64(db))
    errs = {n: rel_err(got[n], want[n]) for n in want}
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL[w.dtype], (n, e)


def test_first_stage_gradient_is_bit_reproducible_and_takes_any_range():
    from paper_2601_15473_amd import libsk as sk
    w = W.Workload("two_range", 900, 256, 320, 2, 32, "bf16", seed=26)
    t = W.generate_two_sided(w)
    l2, k, R = 4, 32, 128
    dt = sk.SK_BF16
    d = {n: to_dev(t.stored[n], w.dtype) for n in ("x", "dY", "B_cat")}
    args = (w.tokens, w.d_in, w.d_out, l2, k)
    need = sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT_FIRST, *args, dt)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    full = torch.empty((w.d_in, R), dtype=torch.float32, device="cuda")
    sk.check(sk.sk_linear_bwd_weight_first(d["x"], d["B_cat"], d["dY"], full, *args, 0, R, dt, ws, need))
    again = torch.full_like(full, float("nan"))
    sk.check(sk.sk_linear_bwd_weight_first(d["x"], d["B_cat"], d["dY"], again, *args, 0, R, dt, ws, need))
    torch.cuda.synchronize()
    assert torch.equal(full.view(torch.int32), again.view(torch.int32))
    # a narrow range in the middle equals those columns of the full result (fp32 sums of the
    # same products; the token split may differ, so to rounding only)
    part = torch.empty((w.d_in, 48), dtype=torch.float32, device="cuda")
    sk.check(sk.sk_linear_bwd_weight_first(d["x"], d["B_cat"], d["dY"], part, *args, 32, 48, dt, ws, need))
    torch.cuda.synchronize()
    assert rel_err(to_f64(part), to_f64(full[:, 32:80])) <= 1e-5
