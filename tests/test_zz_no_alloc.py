"""sk_linear_bwd_weight_noalloc (the entry point for callers that cannot allocate: its
workspace is a fixed device array inside the library) against sk_linear_bwd_weight, through
the C ABI: same kernels, so dU and db must agree bit for bit, and both must meet the
oracle's bar.  Two calls in a row share the array, the second on a smaller input."""
import numpy as np
import pytest
import torch

from oracle import sklinear as O
from paper_2601_15473_amd import workloads as W

pytestmark = pytest.mark.gpu

from skgpu import TOL, DeviceLayer, rel_err, to_f64  # noqa: E402


@pytest.fixture(scope="module")
def sk():
    from paper_2601_15473_amd import libsk
    libsk.sk_set_plan(0)
    yield libsk
    libsk.sk_set_plan(0)


def _noalloc(sk, dev, stream=None, with_db=True):
    return sk.sk_linear_bwd_weight_noalloc(dev.x, dev.S_cat, dev.dY, dev.dU, dev.db if with_db else None,
                                           *dev.args, stream)


def _compare(sk, w, stream=None):
    print(f"case noalloc {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l} k={w.k} {w.dtype}", flush=True)
    t = W.generate(w)
    ref = DeviceLayer(t, sk)
    sk.check(ref.bwd_weight(stream))
    got = DeviceLayer(t, sk)
    sk.check(_noalloc(sk, got, stream))
    torch.cuda.synchronize()
    assert torch.equal(got.dU.view(torch.int32), ref.dU.view(torch.int32))
    assert torch.equal(got.db.view(torch.int32), ref.db.view(torch.int32))
    v = {n: a.astype(np.float64) for n, a in t.value.items()}
    dU = O.grad_factors(v["x"], v["S"], v["dY"]).reshape(w.R, w.d_out)
    db = O.grad_bias(v["dY"])
    errs = dict(dU=rel_err(to_f64(got.dU), dU), db=rel_err(to_f64(got.db), db))
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL[w.dtype], (n, e)
    return t


def test_two_calls_in_a_row_second_one_smaller(sk):
    # BERT-base FFN-up at full size (split token contraction: Z^T, five slabs, column-sum
    # partials all live in the array), then a smaller, ragged layer that reuses its start
    _compare(sk, W.BERT_BASE_FFN_UP)
    t = _compare(sk, W.Workload("bf16_ragged", 333, 208, 176, 3, 16, "bf16", seed=4))
    # ... then fp32, and a call that wants no bias gradient
    _compare(sk, W.Workload("f32_ragged", 77, 48, 80, 3, 16, "f32", seed=1))
    ref = DeviceLayer(t, sk)
    sk.check(ref.bwd_weight())
    nob = DeviceLayer(t, sk)
    sk.check(_noalloc(sk, nob, with_db=False))
    torch.cuda.synchronize()
    assert torch.isnan(nob.db).all()
    assert torch.equal(nob.dU.view(torch.int32), ref.dU.view(torch.int32))


def test_on_a_side_stream_and_largest_benchmark_shape_that_fits(sk):
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    _compare(sk, W.BERT_LARGE_FFN_UP, s)
    _compare(sk, W.scaled(W.BERT_BASE_PROJ[0], tokens=700), s)


def test_too_large_is_an_error_not_a_launch(sk):
    w = W.LLM_MLP
    dt = sk.DTYPES[w.dtype]
    assert sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT, w.tokens, w.d_in, w.d_out, w.l, w.k, dt) \
        > sk.SK_NOALLOC_SCRATCH_BYTES
    dU = torch.full((16,), float("nan"), device="cuda")
    st = sk.sk_linear_bwd_weight_noalloc(dU, dU, dU, dU, None, w.tokens, w.d_in, w.d_out, w.l, w.k, dt, None)
    assert st == sk.SK_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(dU).all()
