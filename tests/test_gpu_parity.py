"""Parity of the HIP path (through the C ABI) with the fp64 oracle, on the GPU.

Bar: max relative error (tests/skgpu.rel_err) <= 1e-4 for fp32 and <= 2e-2 for
bf16 storage with fp32 accumulation -- the tolerances stated for this layer.
The oracle sees the same stored (already rounded) inputs, widened to fp64.
"""
import numpy as np
import pytest
import torch

from oracle import sklinear as O
from paper_2601_15473_amd import workloads as W

pytestmark = pytest.mark.gpu

from skgpu import TOL, DeviceLayer, abs_err_scaled, errors_by_row_blocks, rel_err, to_f64  # noqa: E402


@pytest.fixture(scope="module")
def sk():
    from paper_2601_15473_amd import libsk
    yield libsk
    libsk.sk_set_plan(0)


@pytest.fixture
def tuning(sk):
    """Forces plan parameters for one test: tuning(knob, value); all automatic again afterwards."""
    touched = []

    def force(knob, value):
        touched.append(knob)
        sk.sk_set_tuning(knob, value)
    yield force
    for knob in touched:
        sk.sk_set_tuning(knob, -1)


def oracle_all(t: W.Tensors):
    v = {n: a.astype(np.float64) for n, a in t.value.items()}
    b = v.get("b")
    return dict(
        y=O.forward(v["x"], v["S"], v["U"], b),
        dX=O.grad_input(v["dY"], v["S"], v["U"]),
        dU=O.grad_factors(v["x"], v["S"], v["dY"]).reshape(t.workload.R, t.workload.d_out),
        db=O.grad_bias(v["dY"]),
    )


def check_all(sk, w: W.Workload, plan: int, with_bias=True, single_call=False):
    """The three calls against the oracle; with single_call also sk_linear_bwd (the backward
    pass of the benchmark's timed step) on buffers of its own."""
    print(f"case {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l} k={w.k} "
          f"{w.dtype} plan={plan} bias={with_bias}", flush=True)
    sk.sk_set_plan(plan)
    t = W.generate(w, with_bias=with_bias)
    dev = DeviceLayer(t, sk)
    dev.run_all()
    want = oracle_all(t)
    got = dict(y=to_f64(dev.y), dX=to_f64(dev.dX), dU=to_f64(dev.dU), db=to_f64(dev.db))
    errs = {n: rel_err(got[n], want[n]) for n in want}
    # second figure, so that an error confined to small elements of large rows still shows
    errs2 = {n: abs_err_scaled(got[n], want[n]) for n in want}
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()},
          " max|g-o|/max|o|:", {n: f"{e:.2e}" for n, e in errs2.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL[w.dtype], (n, e)
    for n, e in errs2.items():
        assert e <= TOL[w.dtype], (n, "max|g-o|/max|o|", e)
    if single_call:
        one = DeviceLayer(t, sk)
        sk.check(one.bwd())
        torch.cuda.synchronize()
        for n, g in (("dX", one.dX), ("dU", one.dU), ("db", one.db)):
            e, e2 = rel_err(to_f64(g), want[n]), abs_err_scaled(to_f64(g), want[n])
            print(f"   sk_linear_bwd {n}: {e:.2e}, {e2:.2e}", flush=True)
            assert e <= TOL[w.dtype] and e2 <= TOL[w.dtype], ("sk_linear_bwd", n, e, e2)
    return errs


SMALL = [
    W.TINY,                                                         # config 0 as stated
    W.Workload("f32_ragged", 77, 48, 80, 3, 16, "f32", seed=1),
    W.Workload("f32_multi_tile", 200, 144, 208, 2, 40, "f32", seed=2),
    W.Workload("bf16_one_token", 1, 64, 48, 1, 16, "bf16", seed=3),
    W.Workload("bf16_ragged", 333, 208, 176, 3, 16, "bf16", seed=4),
    W.Workload("bf16_r16", 130, 96, 112, 1, 16, "bf16", seed=5),
    W.scaled(W.BERT_BASE_FFN_UP, tokens=1000),
    W.scaled(W.BERT_LARGE_FFN_UP, tokens=600),
    W.scaled(W.BERT_LARGE_FFN_DOWN, tokens=600),
    W.scaled(W.LLM_MLP, tokens=300),
] + [W.scaled(w, tokens=700) for w in W.BERT_BASE_PROJ] + [
    # the paper's own grid (square 8192 layers); l = 3 makes the 1/l scale inexact
    W.scaled(W.BY_NAME["grid8192_l3_k16"], tokens=200),
    W.scaled(W.BY_NAME["grid8192_l3_k512"], tokens=200),
    # long, ragged contractions (not multiples of the 64-wide k chunk): the first GEMM of a
    # call and the recomputation of Z^T split over them into fp32 slabs
    W.Workload("bf16_long_in_ragged", 300, 2064, 176, 2, 24, "bf16", seed=20),
    W.Workload("bf16_long_out_ragged", 300, 176, 2064, 2, 24, "bf16", seed=21),
    W.Workload("bf16_long_both_r272", 260, 2064, 2064, 2, 136, "bf16", seed=22),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("plan", [2, 1, 3], ids=["two_gemm", "fused", "split_expand"])
def test_parity_small(sk, w, plan):
    check_all(sk, w, plan)


@pytest.mark.parametrize("plan", [2, 1, 3], ids=["two_gemm", "fused", "split_expand"])
def test_no_bias_and_no_dbias(sk, plan):
    w = W.Workload("bf16_nobias", 150, 128, 96, 2, 32, "bf16", seed=6)
    check_all(sk, w, plan, with_bias=False)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd_weight(with_db=False))
    torch.cuda.synchronize()
    assert torch.isnan(dev.db).all()          # untouched when dbias is NULL
    want = oracle_all(t)["dU"]
    assert rel_err(to_f64(dev.dU), want) <= TOL["bf16"]


# Full benchmark sizes, in the automatic plan the benchmark times.
@pytest.mark.parametrize("w", (W.BERT_BASE_FFN_UP,) + W.BERT_BASE_PROJ +
                         (W.BERT_LARGE_FFN_UP, W.BERT_LARGE_FFN_DOWN), ids=lambda w: w.name)
def test_parity_full_size(sk, w):
    check_all(sk, w, 0, single_call=True)


def _kernels_of(sk, dev, calls=("fwd", "bwd_input", "bwd_weight")):
    """Names of the kernels the given calls launch on this layer (per-kernel event timing)."""
    sk.sk_profile_begin(64)
    try:
        for c in calls:
            sk.check(getattr(dev, c)())
    finally:
        names = [r[0] for r in sk.sk_profile_end(64)]
    torch.cuda.synchronize()
    return names


def _check_whole_tensors(sk, w, t, dev):
    """Every element of y, dX, dU and db of a large layer against the oracle, one output at a
    time (each oracle array is dropped before the next is computed)."""
    v = t.value
    S, U = v["S"].astype(np.float64), v["U"].astype(np.float64)
    errs = {}
    x64 = v["x"].astype(np.float64)
    want = O.forward(x64, S, U, v["b"].astype(np.float64))
    errs["y"] = errors_by_row_blocks(dev.y, want)
    del want
    dY64 = v["dY"].astype(np.float64)
    want = O.grad_factors(x64, S, dY64).reshape(w.R, w.d_out)
    errs["dU"] = errors_by_row_blocks(dev.dU, want, block=256)
    del want, x64
    want = O.grad_input(dY64, S, U)
    errs["dX"] = errors_by_row_blocks(dev.dX, want)
    del want
    want = O.grad_bias(dY64)
    errs["db"] = (rel_err(to_f64(dev.db), want), abs_err_scaled(to_f64(dev.db), want))
    print("   errors (rel_err, max|g-o|/max|o|):", {n: f"{a:.2e}, {b:.2e}" for n, (a, b) in errs.items()}, flush=True)
    for n, (a, b) in errs.items():
        assert a <= TOL[w.dtype], (n, a)
        assert b <= TOL[w.dtype], (n, "max|g-o|/max|o|", b)


def test_parity_llm_mlp_full_size(sk):
    """Config 4 (heavy-tailed x, R = 2048) at full size, in the plan the benchmark times:
    every element of all four outputs against one full fp64 pass of the oracle."""
    w = W.LLM_MLP
    print(f"case {w.name} full size, whole tensors", flush=True)
    sk.sk_set_plan(0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    dev.run_all()
    _check_whole_tensors(sk, w, t, dev)
    # the backward pass of the benchmark's timed step: at this size sk_linear_bwd runs the same
    # kernels as the two separate calls, so its results are theirs bit for bit
    one = DeviceLayer(t, sk)
    sk.check(one.bwd())
    torch.cuda.synchronize()
    assert torch.equal(one.dX.view(torch.int16), dev.dX.view(torch.int16))
    assert torch.equal(one.dU.view(torch.int32), dev.dU.view(torch.int32))
    assert torch.equal(one.db.view(torch.int32), dev.db.view(torch.int32))


def test_parity_big_tile_paths_mid_size(sk):
    """The code only shapes like config 4 reach, on a layer small enough to check quickly and
    ragged in every dimension: eight-wave 256 x 256 tiles walked by a crew of work-groups
    (five or six tiles each), a factor gradient with more tiles than CUs but fewer than two
    rounds -- a first round of whole-token tiles straight into dU, the remaining tile columns
    split over the tokens, their slabs summed by the column-range reduction -- and the bias
    gradient's column sums riding in that second launch.  Whole tensors against the oracle."""
    w = W.Workload("bf16_big_tile_paths", 8203, 1040, 10480, 8, 256, "bf16", x_dist="student_t3", seed=40)
    print(f"case {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l} k={w.k}", flush=True)
    sk.sk_set_plan(0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    dev.run_all()
    _check_whole_tensors(sk, w, t, dev)
    names = _kernels_of(sk, DeviceLayer(t, sk))
    print("   kernels:", names, flush=True)
    assert any(n.startswith("gemm_bf16_crew_kernel<256, 256, 2, 4, true, false, bf16") for n in names)   # Z.U
    assert any(n.startswith("gemm_bf16_crew_kernel<256, 256, 2, 4, true, true, bf16") for n in names)    # dY.U^T
    assert any(n.startswith("gemm_bf16_with_colsum_kernel") for n in names)
    assert "reduce_splits_2d_kernel" in names


def test_outputs_past_two_gib_sampled(sk):
    """A token count that puts y and dY past 2^31 bytes (byte offsets no longer fit 32 bits
    anywhere but inside one tile): c1's layer at 360 000 tokens, checked on sampled token
    rows of y and dX (first, last and random ones) and sampled columns of dU and db."""
    # (a seeded block of 36 000 tokens repeated ten times: drawing 1.4e9 fresh normals on
    # the host would take minutes and add nothing to the check)
    block = W.generate(W.scaled(W.BERT_BASE_FFN_UP, tokens=36_000, seed=31))
    w = W.scaled(block.workload, tokens=360_000)
    assert w.tokens * w.d_out * 2 > 2 ** 31
    print(f"case {w.name} T={w.tokens} (outputs past 2 GiB, sampled)", flush=True)
    sk.sk_set_plan(0)
    rep = lambda d: {n: (np.tile(a, (10, 1)) if n in ("x", "dY") else a) for n, a in d.items()}  # noqa: E731
    t = W.Tensors(w, rep(block.stored), rep(block.value))
    dev = DeviceLayer(t, sk)
    dev.run_all()
    r = np.random.default_rng(7)
    rows = np.sort(r.choice(w.tokens, 64, replace=False))
    rows[0], rows[-1] = 0, w.tokens - 1
    rows[1], rows[-2] = 2 ** 31 // (w.d_out * 2) - 1, 2 ** 31 // (w.d_out * 2) + 1   # either side of 2 GiB in y
    rows = np.unique(rows)
    cols = np.sort(r.choice(w.d_out, 24, replace=False))
    cols[0], cols[-1] = 0, w.d_out - 1
    v = t.value
    S, U = v["S"].astype(np.float64), v["U"].astype(np.float64)
    y = O.forward(v["x"][rows].astype(np.float64), S, U, v["b"].astype(np.float64))
    dX = O.grad_input(v["dY"][rows].astype(np.float64), S, U)
    dYc = v["dY"][:, cols].astype(np.float64)
    dU = O.grad_factors(v["x"].astype(np.float64), S, dYc).reshape(w.R, len(cols))
    db = O.grad_bias(dYc)
    rows_t, cols_t = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
    errs = dict(y=rel_err(to_f64(dev.y[rows_t]), y), dX=rel_err(to_f64(dev.dX[rows_t]), dX),
                dU=rel_err(to_f64(dev.dU[:, cols_t]), dU), db=rel_err(to_f64(dev.db[cols_t]), db))
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL["bf16"], (n, e)
    # nothing left unwritten anywhere (the buffers start as NaN)
    assert torch.isfinite(dev.y.view(torch.int16).view(torch.bfloat16)[-4096:].float()).all()
    assert not torch.isnan(dev.dX.float().sum()) and not torch.isnan(dev.y[:100000].float().sum())
    assert not torch.isnan(dev.y[100000:].float().sum())


BWD_CASES = [
    W.Workload("bf16_long_both_r272", 260, 2064, 2064, 2, 136, "bf16", seed=22),   # split first GEMMs: no shared launches
    W.scaled(W.BY_NAME["grid8192_l1_k16"], tokens=300),                             # split Z^T recomputation
    W.scaled(W.BERT_BASE_FFN_UP, tokens=1000),        # shared launches (R = 128, long first contraction)
    W.BERT_BASE_FFN_UP,
    W.scaled(W.BERT_BASE_PROJ[0], tokens=700),        # R = 32: 64 x 64 tiles
    W.BERT_BASE_PROJ[2],
    W.Workload("bf16_ragged", 333, 208, 176, 3, 16, "bf16", seed=4),
    W.Workload("bf16_one_token", 1, 64, 48, 1, 16, "bf16", seed=3),
    W.scaled(W.BERT_LARGE_FFN_UP, tokens=600),        # wide sketch, too few tokens for the shared launches
    W.scaled(W.BERT_LARGE_FFN_UP, tokens=5000),       # wide sketch: shared launches (128 x 128 tiles)
    W.scaled(W.BERT_LARGE_FFN_DOWN, tokens=4100),     # ... with a split token contraction
    W.scaled(W.BERT_BASE_PROJ[3], tokens=700),        # R = 256, too few tokens for the shared launches
    W.BERT_BASE_PROJ[3],                              # R = 256: shared launches on 64 x 64 / 128 x 64 tiles
    W.BERT_BASE_PROJ[4],                              # R = 384
    W.Workload("f32_ragged", 77, 48, 80, 3, 16, "f32", seed=1),
]


@pytest.mark.parametrize("w", BWD_CASES, ids=lambda w: f"{w.name}_T{w.tokens}")
def test_single_call_backward(sk, w):
    """sk_linear_bwd against the oracle, and against the two separate calls: dU and db bit
    for bit, dX to the tolerance (its fp32 partial sums may be ordered differently)."""
    print(f"case bwd {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l} k={w.k} {w.dtype}", flush=True)
    sk.sk_set_plan(0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd())
    torch.cuda.synchronize()
    want = oracle_all(t)
    got = dict(dX=to_f64(dev.dX), dU=to_f64(dev.dU), db=to_f64(dev.db))
    errs = {n: rel_err(got[n], want[n]) for n in got}
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL[w.dtype], (n, e)
    sep = DeviceLayer(t, sk)
    sk.check(sep.bwd_input())
    sk.check(sep.bwd_weight())
    torch.cuda.synchronize()
    one_pass = any("bwd_narrow" in n for n in _kernels_of(sk, DeviceLayer(t, sk), ("bwd",)))
    if one_pass:   # per-token-tile partial sums: another summation order than the separate call's
        assert rel_err(to_f64(dev.dU), to_f64(sep.dU)) <= TOL[w.dtype]
        assert rel_err(to_f64(dev.db), to_f64(sep.db)) <= TOL[w.dtype]
    else:
        assert torch.equal(dev.dU.view(torch.int32), sep.dU.view(torch.int32))
        assert torch.equal(dev.db.view(torch.int32), sep.db.view(torch.int32))
    assert rel_err(to_f64(dev.dX), to_f64(sep.dX)) <= TOL[w.dtype]
    # no bias gradient wanted
    nob = DeviceLayer(t, sk)
    sk.check(nob.bwd(with_db=False))
    torch.cuda.synchronize()
    assert torch.isnan(nob.db).all()
    assert torch.equal(nob.dU.view(torch.int32), dev.dU.view(torch.int32))


NARROW_CASES = [
    # (workload, forced tokens per work-group or None): the one-pass schedule where the planner
    # takes it by itself (one round of token tiles: 32-token tiles up to 8192 tokens, 64-token
    # tiles up to 16384) and forced onto small cases, both tile heights: ragged token tiles, a
    # single chunk, chunk counts on both sides of a pass of eight (out = 1024 | 1040 | 2320), R
    # below the kernel's width, the longest input it takes, a second round of work-groups
    (W.BERT_BASE_PROJ[0], None),
    (W.scaled(W.BERT_BASE_PROJ[0], tokens=16384), None),
    (W.Workload("narrow_many_tiles", 15000, 96, 160, 1, 32, "bf16", seed=36), None),
    (W.Workload("narrow_two_rounds", 20000, 96, 160, 1, 32, "bf16", seed=36), 64),
    (W.scaled(W.BERT_BASE_PROJ[0], tokens=1237), 32),
    (W.scaled(W.BERT_BASE_PROJ[0], tokens=1237), 64),
    (W.Workload("narrow_r16", 3333, 144, 336, 1, 16, "bf16", seed=37), 32),
    (W.Workload("narrow_one_chunk", 130, 64, 48, 1, 16, "bf16", seed=32), 64),
    (W.Workload("narrow_one_chunk", 130, 64, 48, 1, 16, "bf16", seed=32), 32),
    (W.Workload("narrow_longest_in", 200, 848, 208, 2, 16, "bf16", seed=33), 32),
    (W.Workload("narrow_longest_in", 200, 848, 208, 2, 16, "bf16", seed=33), 64),
    (W.Workload("narrow_full_pass", 77, 400, 1024, 1, 32, "bf16", seed=34), 64),
    (W.Workload("narrow_pass_and_a_bit", 150, 112, 1040, 1, 32, "bf16", seed=38), 32),
    (W.Workload("narrow_three_passes", 100, 64, 2320, 2, 16, "bf16", seed=39), 64),
    (W.Workload("narrow_three_passes", 100, 64, 2320, 2, 16, "bf16", seed=39), 32),
    (W.Workload("narrow_one_token", 1, 16, 16, 1, 16, "bf16", seed=35), 32),
]


@pytest.mark.parametrize("w,forced", NARROW_CASES, ids=lambda v: f"{v.name}_T{v.tokens}" if hasattr(v, "name") else (f"tm{v}" if v else "auto"))
def test_one_pass_backward_for_narrow_sketches(sk, tuning, w, forced):
    """sk_linear_bwd's one-pass schedule (a kernel that reads x and dY once, writes dX and
    leaves a slab of dU and db per token tile, then the sum of the slabs): the kernel runs --
    by the planner's own choice on the large cases, forced on the small ones -- and every
    element of dX, dU and db agrees with the oracle."""
    print(f"case narrow {w.name} T={w.tokens} in={w.d_in} out={w.d_out} l={w.l} k={w.k} forced={forced}", flush=True)
    sk.sk_set_plan(0)
    if forced:
        tuning(sk.SK_TUNE_NARROW_BWD, forced)
    t = W.generate(w)
    names = _kernels_of(sk, DeviceLayer(t, sk), ("bwd",))
    assert len(names) == 2 and "bwd_narrow_kernel" in names[0] and "reduce_tiles" in names[1], names
    if forced:
        assert names[0] == f"bwd_narrow_kernel<{forced // 32}>", names
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd())
    torch.cuda.synchronize()
    want = oracle_all(t)
    got = dict(dX=to_f64(dev.dX), dU=to_f64(dev.dU), db=to_f64(dev.db))
    errs = {n: rel_err(got[n], want[n]) for n in got}
    print("   errors:", {n: f"{e:.2e}" for n, e in errs.items()}, flush=True)
    for n, e in errs.items():
        assert e <= TOL[w.dtype], (n, e)
    again = DeviceLayer(t, sk)
    sk.check(again.bwd())
    torch.cuda.synchronize()
    for a, b in ((dev.dX, again.dX), (dev.dU, again.dU), (dev.db, again.db)):   # bit-reproducible
        assert torch.equal(a.view(torch.int16 if a.element_size() == 2 else torch.int32),
                           b.view(torch.int16 if b.element_size() == 2 else torch.int32))


def _random_shapes(n, seed):
    r = np.random.default_rng(seed)
    out = []
    for i in range(n):
        l = int(r.integers(1, 5))
        k = int(r.choice([16, 32, 48, 64, 96]))
        out.append(W.Workload(f"rnd{i}", int(r.integers(1, 900)), 16 * int(r.integers(1, 40)),
                              16 * int(r.integers(1, 40)), l, k, "f32" if i % 6 == 5 else "bf16", seed=100 + i))
    return out


@pytest.mark.parametrize("w", _random_shapes(24, 2024), ids=lambda w: f"{w.name}_T{w.tokens}_{w.d_in}x{w.d_out}_l{w.l}k{w.k}_{w.dtype}")
def test_random_shapes(sk, w):
    """Seeded random shapes (ragged token counts, every multiple of 16 for the feature sizes,
    sketch widths on both sides of every plan boundary), automatic plan, three calls and
    the single-call backward."""
    check_all(sk, w, 0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd())
    torch.cuda.synchronize()
    want = oracle_all(t)
    for n, got in (("dX", dev.dX), ("dU", dev.dU), ("db", dev.db)):
        assert rel_err(to_f64(got), want[n]) <= TOL[w.dtype], n


def test_forced_big_tiles(sk, tuning):
    """The large-shape code paths (big tiles, the bias gradient from its own kernel)
    on a shape small enough for a full oracle pass."""
    w = W.Workload("bf16_forced_paths", 700, 320, 592, 2, 72, "bf16", seed=10)
    for tile, wtile in ((7, 7), (0, 5), (5, 1), (6, 2)):
        tuning(sk.SK_TUNE_TILE, tile)
        tuning(sk.SK_TUNE_WTILE, wtile)
        check_all(sk, w, 2)


TALL_CASES = [
    W.Workload("bf16_ragged", 333, 208, 176, 3, 16, "bf16", seed=4),          # R = 48, ragged last tile
    W.Workload("bf16_one_token", 1, 64, 48, 1, 16, "bf16", seed=3),
    W.scaled(W.BERT_BASE_FFN_UP, tokens=1000),                                # R = 128
    W.scaled(W.BERT_BASE_PROJ[1], tokens=700),                                # R = 64
    W.Workload("bf16_r128_ragged", 129, 272, 400, 2, 64, "bf16", seed=12),    # one row past a tile
]


@pytest.mark.parametrize("w", TALL_CASES, ids=lambda w: f"{w.name}_T{w.tokens}")
@pytest.mark.parametrize("plan", [1, 3], ids=["fused", "split_expand"])
def test_tall_token_tiles_forced(sk, tuning, w, plan):
    """The 128-row token tiles of the narrow kernels (picked by themselves only from 32768
    tokens on), forced onto shapes small and ragged enough for a full oracle pass: three
    calls and the single-call backward."""
    tuning(sk.SK_TUNE_BM, 128)
    check_all(sk, w, plan)
    sk.sk_set_plan(0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd())
    torch.cuda.synchronize()
    want = oracle_all(t)
    for n, got in (("dX", dev.dX), ("dU", dev.dU), ("db", dev.db)):
        assert rel_err(to_f64(got), want[n]) <= TOL[w.dtype], n


def test_tall_token_tiles_by_themselves(sk):
    """Past 128 x 256 tokens the automatic plan takes the 128-row tiles: a narrow layer at
    32768 + 77 tokens (ragged last tile), full oracle pass."""
    w = W.Workload("bf16_many_tokens", 32768 + 77, 128, 384, 2, 32, "bf16", seed=13)
    check_all(sk, w, 0)
    w = W.Workload("bf16_many_tokens_r128", 32768 + 1, 96, 256, 2, 64, "bf16", seed=14)
    check_all(sk, w, 0)


EXTREME_CASES = [
    (70, 65536, 16, 1, 16), (70, 16, 65536, 1, 16), (33000, 16, 16, 1, 16), (10, 2048, 2048, 8, 256),
    (1, 16, 16, 1, 16), (4097, 48, 33040, 3, 16), (129, 30000, 272, 1, 272), (65, 4112, 4112, 2, 1024),
]


@pytest.mark.parametrize("shape", EXTREME_CASES, ids=lambda c: "T%d_%dx%d_l%dk%d" % c)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_extreme_aspect_ratios(sk, shape, dtype):
    """Shapes at the far ends of what the planner sees: one token, 65536-wide sides against
    16-wide ones, a sketch as wide as the layer, a contraction 30000 long."""
    T, d_in, d_out, l, k = shape
    w = W.Workload("extreme", T, d_in, d_out, l, k, dtype, seed=500 + EXTREME_CASES.index(shape))
    check_all(sk, w, 0)
    t = W.generate(w)
    dev = DeviceLayer(t, sk)
    sk.check(dev.bwd())
    torch.cuda.synchronize()
    want = oracle_all(t)
    for n, got in (("dX", dev.dX), ("dU", dev.dU), ("db", dev.db)):
        assert rel_err(to_f64(got), want[n]) <= TOL[w.dtype], n


def test_bit_reproducible(sk):
    """The token reduction of dU/db runs in a fixed order: two runs agree bit for bit."""
    sk.sk_set_plan(0)
    t = W.generate(W.scaled(W.BERT_BASE_FFN_UP, tokens=2000))
    dev = DeviceLayer(t, sk)
    dev.run_all()
    first = [a.clone() for a in (dev.y, dev.dX, dev.dU, dev.db)]
    for a in (dev.y, dev.dX, dev.dU, dev.db):
        a.fill_(float("nan"))
    dev.run_all()
    for a, b in zip(first, (dev.y, dev.dX, dev.dU, dev.db)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_runs_on_a_side_stream(sk):
    sk.sk_set_plan(0)
    t = W.generate(W.Workload("bf16_stream", 500, 256, 320, 2, 32, "bf16", seed=8))
    dev = DeviceLayer(t, sk)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    for st in (dev.fwd(s), dev.bwd_input(s), dev.bwd_weight(s)):
        sk.check(st)
    s.synchronize()
    want = oracle_all(t)
    got = dict(y=to_f64(dev.y), dX=to_f64(dev.dX), dU=to_f64(dev.dU), db=to_f64(dev.db))
    for n in want:
        assert rel_err(got[n], want[n]) <= TOL["bf16"], n


def test_workspace_too_small_is_an_error_not_a_launch(sk):
    t = W.generate(W.Workload("bf16_ws", 64, 64, 64, 1, 16, "bf16", seed=9))
    dev = DeviceLayer(t, sk)
    sk.sk_set_plan(2)
    st = sk.sk_linear_fwd(dev.x, dev.S_cat, dev.U_cat, dev.b, dev.y, *dev.args, dev.ws, 8, None)
    assert st == sk.SK_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(dev.y.float()).all()
