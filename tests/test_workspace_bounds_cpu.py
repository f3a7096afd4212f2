"""Host-side guard of the planner's buffer arithmetic, without a GPU.

In trace mode (include/sk_debug.h) the entry points plan as usual but launch nothing; each
kernel they would launch reports the byte ranges it reads and writes.  For many seeded
shapes, every entry point, every plan and forced plan parameters, each range must lie
wholly inside one of the caller's buffers -- the workspace being exactly as large as
sk_linear_workspace_bytes says -- inputs are never written, and a kernel never writes a
range that it (or the other half of a shared launch) also touches elsewhere."""
import os

import numpy as np
import pytest

from paper_2601_15473_amd import libsk as sk

N_SHAPES = int(os.environ.get("SK_TRACE_SHAPES", "100000"))
SPACING = 1 << 44      # made-up device addresses, far apart; never dereferenced


def _log_int(r, lo, hi):
    return int(round(np.exp(r.uniform(np.log(lo), np.log(hi)))))


def _shape(r):
    T = _log_int(r, 1, 70000)
    d_in = 16 * _log_int(r, 1, 1024)
    d_out = 16 * _log_int(r, 1, 1024)
    l = int(r.integers(1, 9))
    # R = l k a multiple of 16, up to 4096
    k = 16 * _log_int(r, 1, max(1, 256 // l)) // (16 if l % 16 == 0 else 1)
    while (l * k) % 16:
        k += 1
    dtype = sk.SK_BF16 if r.random() < 0.8 else sk.SK_F32
    return T, d_in, d_out, l, k, dtype


class Buffers:
    def __init__(self, T, d_in, d_out, l, k, dtype, nc):
        e = 2 if dtype == sk.SK_BF16 else 4
        R = l * k
        sizes = dict(x=T * d_in * e, dY=T * d_out * e, S=d_in * R * e, U=R * d_out * e, b=d_out * e,
                     y=T * d_out * e, dX=T * d_in * e, dU=R * d_out * 4, db=d_out * 4, dA=d_in * nc * 4)
        self.size = sizes
        self.base = {n: (i + 1) * SPACING for i, n in enumerate(sizes)}
        self.base["ws"] = (len(sizes) + 1) * SPACING

    def check(self, trace, launches, ws_bytes, outputs, what):
        assert launches >= 1, what
        self.size["ws"] = ws_bytes
        per_launch = {}
        for addr, nbytes, write, launch in trace:
            assert nbytes > 0, what
            owner = None
            for n, base in self.base.items():
                if base <= addr < base + SPACING:
                    owner = n
                    break
            assert owner is not None, (what, hex(addr))
            off = addr - self.base[owner]
            assert off + nbytes <= self.size[owner], \
                (what, f"launch {launch}: {'write' if write else 'read'} of {owner}[{off}:{off + nbytes}] "
                       f"past its {self.size[owner]} bytes")
            if write:
                assert owner == "ws" or owner in outputs, (what, f"launch {launch} writes {owner}")
            per_launch.setdefault(launch, []).append((addr, addr + nbytes, write))
        for launch, ranges in per_launch.items():
            for i, (a0, a1, w) in enumerate(ranges):
                if not w:
                    continue
                for j, (b0, b1, _) in enumerate(ranges):
                    if i != j:
                        assert a1 <= b0 or b1 <= a0, (what, f"launch {launch}: a written range overlaps another")


def _calls(buf, args, nc, c0):
    B = buf.base
    ws = B["ws"]
    return {
        sk.SK_OP_FWD: (("y",), lambda n: sk.sk_linear_fwd(B["x"], B["S"], B["U"], B["b"], B["y"], *args, ws, n)),
        sk.SK_OP_BWD_INPUT: (("dX",), lambda n: sk.sk_linear_bwd_input(B["dY"], B["S"], B["U"], B["dX"], *args, ws, n)),
        sk.SK_OP_BWD_WEIGHT: (("dU", "db"), lambda n: sk.sk_linear_bwd_weight(
            B["x"], B["S"], B["dY"], B["dU"], B["db"], *args, ws, n)),
        sk.SK_OP_BWD: (("dX", "dU", "db"), lambda n: sk.sk_linear_bwd(
            B["x"], B["dY"], B["S"], B["U"], B["dX"], B["dU"], B["db"], *args, ws, n)),
        sk.SK_OP_BWD_WEIGHT_FIRST: (("dA",), lambda n: sk.sk_linear_bwd_weight_first(
            B["x"], B["U"], B["dY"], B["dA"], *args[:5], c0, nc, args[5], ws, n)),
    }


def _run_shape(r, shape, plan, forced):
    T, d_in, d_out, l, k, dtype = shape
    R = l * k
    nc = 16 * int(r.integers(1, R // 16 + 1))
    c0 = 16 * int(r.integers(0, (R - nc) // 16 + 1))
    buf = Buffers(T, d_in, d_out, l, k, dtype, nc)
    sk.sk_set_plan(plan)
    for knob, value in forced:
        sk.sk_set_tuning(knob, value)
    try:
        for op, (outputs, call) in _calls(buf, shape, nc, c0).items():
            need = sk.sk_linear_workspace_bytes(op, *shape)
            assert need != 2 ** 64 - 1
            what = (shape, f"op {op} plan {plan} forced {forced} cols {c0}+{nc}")
            sk.sk_trace_begin()
            try:
                st = call(need)
            finally:
                trace, launches = sk.sk_trace_end()
            assert st == sk.SK_OK, (what, sk.sk_status_string(st))
            buf.check(trace, launches, need, outputs, what)
    finally:
        for knob, _ in forced:
            sk.sk_set_tuning(knob, -1)
        sk.sk_set_plan(0)


def _forced(r):
    """A few forced plan parameters (often none)."""
    if r.random() < 0.6:
        return ()
    out = []
    for knob, lo, hi in ((sk.SK_TUNE_TILE, 0, 8), (sk.SK_TUNE_WTILE, 0, 8), (sk.SK_TUNE_WSPLITS, 1, 33),
                         (sk.SK_TUNE_SLICES, 1, 40), (sk.SK_TUNE_STILE, 1, 5), (sk.SK_TUNE_SSPLITS, 1, 10)):
        if r.random() < 0.3:
            out.append((knob, int(r.integers(lo, hi))))
    if r.random() < 0.3:
        out.append((sk.SK_TUNE_BM, int(r.choice([64, 128]))))
    if r.random() < 0.3:
        out.append((sk.SK_TUNE_NARROW_BWD, int(r.choice([0, 1, 32, 64]))))
    return tuple(out)


def test_every_access_of_every_plan_stays_inside_the_buffers():
    r = np.random.default_rng(20260115)
    for i in range(N_SHAPES):
        _run_shape(r, _shape(r), int(r.integers(0, 4)), _forced(r))


BENCH_SHAPES = [
    (64, 256, 256, 1, 16, sk.SK_F32), (4096, 768, 3072, 2, 64, sk.SK_BF16), (4096, 768, 768, 2, 192, sk.SK_BF16),
    (8192, 1024, 4096, 4, 128, sk.SK_BF16), (8192, 4096, 1024, 4, 128, sk.SK_BF16),
    (16384, 4096, 11008, 8, 256, sk.SK_BF16), (4096, 8192, 8192, 3, 512, sk.SK_BF16),
    (360000, 768, 3072, 2, 64, sk.SK_BF16), (1, 16, 16, 1, 16, sk.SK_BF16), (65, 4112, 4112, 2, 1024, sk.SK_F32),
]


@pytest.mark.parametrize("shape", BENCH_SHAPES, ids=lambda s: "T%d_%dx%d_l%dk%d_%d" % s)
def test_benchmark_and_extreme_shapes_every_plan_and_tile(shape):
    r = np.random.default_rng(7)
    for plan in range(4):
        _run_shape(r, shape, plan, ())
        for tile in range(8):
            _run_shape(r, shape, plan, ((sk.SK_TUNE_TILE, tile), (sk.SK_TUNE_WTILE, tile)))
        for bm in (64, 128):
            _run_shape(r, shape, plan, ((sk.SK_TUNE_BM, bm), (sk.SK_TUNE_SLICES, 3)))


def test_one_pass_backward_stays_inside_the_buffers():
    """sk_linear_bwd's one-pass schedule for narrow sketches (two launches: the pass, then the
    sum of the token tiles' slabs), chosen by the planner on the first shape and forced on
    the others: ragged tokens, one chunk, several flush passes, the longest input."""
    r = np.random.default_rng(11)
    shapes = [(16384, 768, 768, 2, 16, sk.SK_BF16), (4096, 768, 768, 2, 16, sk.SK_BF16), (8193, 96, 160, 1, 32, sk.SK_BF16),
              (1237, 768, 768, 2, 16, sk.SK_BF16), (130, 64, 48, 1, 16, sk.SK_BF16),
              (200, 848, 208, 2, 16, sk.SK_BF16), (100, 64, 2320, 2, 16, sk.SK_BF16),
              (1, 16, 16, 1, 16, sk.SK_BF16), (70000, 848, 4096, 1, 32, sk.SK_BF16)]
    for i, shape in enumerate(shapes):
        forced = () if i < 3 else ((sk.SK_TUNE_NARROW_BWD, (1, 32, 64)[i % 3]),)
        for knob, value in forced:
            sk.sk_set_tuning(knob, value)
        try:
            B = Buffers(*shape, 16).base
            sk.sk_trace_begin()
            try:
                st = sk.sk_linear_bwd(B["x"], B["dY"], B["S"], B["U"], B["dX"], B["dU"], B["db"], *shape,
                                      B["ws"], sk.sk_linear_workspace_bytes(sk.SK_OP_BWD, *shape))
            finally:
                _, launches = sk.sk_trace_end()
            assert st == sk.SK_OK and launches == 2, (shape, st, launches)
        finally:
            for knob, _ in forced:
                sk.sk_set_tuning(knob, -1)
        _run_shape(r, shape, 0, forced)
    # not taken for wider sketches, longer inputs or other plans
    for shape, plan in (((16384, 768, 768, 1, 64, sk.SK_BF16), 0), ((16384, 864, 768, 1, 32, sk.SK_BF16), 0),
                        ((16384, 768, 768, 1, 32, sk.SK_F32), 0), ((16384, 768, 768, 1, 32, sk.SK_BF16), 2)):
        sk.sk_set_plan(plan)
        sk.sk_set_tuning(sk.SK_TUNE_NARROW_BWD, 1)
        try:
            B = Buffers(*shape, 16).base
            sk.sk_trace_begin()
            try:
                st = sk.sk_linear_bwd(B["x"], B["dY"], B["S"], B["U"], B["dX"], B["dU"], B["db"], *shape,
                                      B["ws"], sk.sk_linear_workspace_bytes(sk.SK_OP_BWD, *shape))
            finally:
                _, launches = sk.sk_trace_end()
            assert st == sk.SK_OK and launches > 2, (shape, plan, launches)
        finally:
            sk.sk_set_tuning(sk.SK_TUNE_NARROW_BWD, -1)
            sk.sk_set_plan(0)


def test_trace_mode_launches_nothing_and_ends_cleanly():
    sk.sk_trace_begin()
    st = sk.sk_linear_fwd(0x1000, 0x2000, 0x3000, None, 0x4000, 64, 64, 64, 1, 16, sk.SK_BF16, None, 0)
    trace, launches = sk.sk_trace_end()
    assert st == sk.SK_OK and launches == 1           # the fused kernel needs no workspace
    assert {a for a, _, w, _ in trace if w} == {0x4000}
    assert sk.sk_trace_end() == ([], 0)               # no trace open: nothing recorded
    assert sk.sk_set_tuning(99, 1) == -2 ** 31
    assert sk.sk_set_tuning(sk.SK_TUNE_BM, 128) == -1
    assert sk.sk_set_tuning(sk.SK_TUNE_BM, -5) == 128
