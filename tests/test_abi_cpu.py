"""The C ABI without a GPU: the library loads, exports what include/sk.h
declares, and rejects bad arguments before touching HIP."""
import os
import re

import pytest

from paper_2601_15473_amd import libsk as sk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000      # a fake, 16-byte aligned device address: never dereferenced on these paths
ARGS = (64, 64, 64, 1, 16, sk.SK_BF16)


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "sk.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sk_[a-z_]+)\s*\(", hdr))
    assert declared == set(sk.EXPORTS)
    for name in declared:
        assert hasattr(sk._lib, name), name
    # the testing / measurement aids have a header of their own
    dbg = open(os.path.join(ROOT, "include", "sk_debug.h")).read()
    dbg = re.sub(r"/\*.*?\*/", "", dbg, flags=re.S)
    declared = set(re.findall(r"\b(sk_[a-z_]+)\s*\(", dbg))
    assert declared == set(sk.DEBUG_EXPORTS)
    for name in declared:
        assert hasattr(sk._lib, name), name


def test_status_strings():
    for s in range(5):
        assert sk.sk_status_string(s).startswith(("SK_OK", "SK_ERR"))
    assert "unknown" in sk.sk_status_string(99)
    assert sk.sk_last_hip_error() == ""


def test_null_and_misaligned_pointers():
    assert sk.sk_linear_fwd(None, P, P, P, P, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_fwd(P, P, P, None, None, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_fwd(P + 2, P, P, P, P, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_fwd(P, P, P, P + 8, P, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_bwd_input(P, None, P, P, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_bwd_input(P, P, P, P + 4, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_bwd_weight(P, P, P, None, P, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG
    assert sk.sk_linear_bwd_weight(P, P, P, P, P + 4, *ARGS, P, 1 << 20) == sk.SK_ERR_INVALID_ARG


@pytest.mark.parametrize("bad, want", [
    ((0, 64, 64, 1, 16, sk.SK_BF16), sk.SK_ERR_INVALID_ARG),
    ((64, -16, 64, 1, 16, sk.SK_BF16), sk.SK_ERR_INVALID_ARG),
    ((64, 64, 64, 0, 16, sk.SK_BF16), sk.SK_ERR_INVALID_ARG),
    ((64, 64, 64, 1, 0, sk.SK_F32), sk.SK_ERR_INVALID_ARG),
    ((64, 72, 64, 1, 16, sk.SK_BF16), sk.SK_ERR_UNSUPPORTED),   # in not a multiple of 16
    ((64, 64, 40, 1, 16, sk.SK_BF16), sk.SK_ERR_UNSUPPORTED),
    ((64, 64, 64, 3, 5, sk.SK_F32), sk.SK_ERR_UNSUPPORTED),     # l*k = 15
    ((64, 64, 64, 1, 16, 7), sk.SK_ERR_UNSUPPORTED),            # unknown dtype
])
def test_bad_shapes(bad, want):
    assert sk.sk_linear_fwd(P, P, P, P, P, *bad, P, 1 << 30) == want
    assert sk.sk_linear_bwd_input(P, P, P, P, *bad, P, 1 << 30) == want
    assert sk.sk_linear_bwd_weight(P, P, P, P, P, *bad, P, 1 << 30) == want
    for op in (0, 1, 2):
        assert sk.sk_linear_workspace_bytes(op, *bad) == 2 ** 64 - 1
    assert sk.sk_linear_workspace_bytes(9, *ARGS) == 2 ** 64 - 1


def test_workspace_query_and_check():
    sk.sk_set_plan(2)
    try:
        for dt, e in ((sk.SK_BF16, 2), (sk.SK_F32, 4)):
            a = (1000, 768, 3072, 2, 64, dt)
            mid = 1000 * 128 * e
            for op in (sk.SK_OP_FWD, sk.SK_OP_BWD_INPUT):
                ws = sk.sk_linear_workspace_bytes(op, *a)
                # the intermediate, plus at most eight fp32 slabs of a split first contraction
                assert ws >= mid and ws % 256 == 0 and ws <= mid + 8 * 4 * 1000 * 128 + 512
            assert sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT, *a) >= mid
        need = sk.sk_linear_workspace_bytes(sk.SK_OP_FWD, *ARGS)
        assert sk.sk_linear_fwd(P, P, P, P, P, *ARGS, P, need - 1) == sk.SK_ERR_WORKSPACE
        assert sk.sk_linear_fwd(P, P, P, P, P, *ARGS, None, 0) == sk.SK_ERR_WORKSPACE
        assert sk.sk_linear_bwd_input(P, P, P, P, *ARGS, P, need - 1) == sk.SK_ERR_WORKSPACE
        needw = sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT, *ARGS)
        assert sk.sk_linear_bwd_weight(P, P, P, P, P, *ARGS, P, needw - 1) == sk.SK_ERR_WORKSPACE
    finally:
        sk.sk_set_plan(0)


def test_set_plan():
    assert sk.sk_set_plan(4) == -1 and sk.sk_set_plan(-1) == -1
    prev = sk.sk_set_plan(2)
    assert sk.sk_set_plan(prev) == 2


def test_check_raises():
    with pytest.raises(sk.SkError) as e:
        sk.check(sk.SK_ERR_UNSUPPORTED)
    assert e.value.status == sk.SK_ERR_UNSUPPORTED
    sk.check(sk.SK_OK)


def test_first_stage_gradient_argument_checks():
    T, i, o, l, k, dt = ARGS
    R = l * k
    f = sk.sk_linear_bwd_weight_first
    big = 1 << 30
    assert f(None, P, P, P, T, i, o, l, k, 0, R, dt, P, big) == sk.SK_ERR_INVALID_ARG
    assert f(P, P, P, P + 4, T, i, o, l, k, 0, R, dt, P, big) == sk.SK_ERR_INVALID_ARG
    for c0, nc in ((0, 0), (8, 16), (0, 24), (16, R), (-16, 16)):       # empty, misaligned, past the end
        assert f(P, P, P, P, T, i, o, l, k, c0, nc, dt, P, big) == sk.SK_ERR_INVALID_ARG, (c0, nc)
    assert f(P, P, P, P, T, i, o, l, k, 0, R, 7, P, big) == sk.SK_ERR_UNSUPPORTED
    need = sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT_FIRST, *ARGS)
    assert 0 < need < 2 ** 63
    assert f(P, P, P, P, T, i, o, l, k, 0, R, dt, P, need - 1) == sk.SK_ERR_WORKSPACE
    assert f(P, P, P, P, T, i, o, l, k, 0, R, dt, None, 0) == sk.SK_ERR_WORKSPACE


def test_single_call_backward_argument_checks_and_workspace():
    f = sk.sk_linear_bwd
    big = 1 << 30
    assert f(None, P, P, P, P, P, P, *ARGS, P, big) == sk.SK_ERR_INVALID_ARG
    assert f(P, P, P, P, P + 8, P, P, *ARGS, P, big) == sk.SK_ERR_INVALID_ARG
    assert f(P, P, P, P, P, P, None, 64, 64, 60, 1, 16, sk.SK_BF16, P, big) == sk.SK_ERR_UNSUPPORTED
    for a in (ARGS, (4096, 768, 3072, 2, 64, sk.SK_BF16), (8192, 1024, 4096, 4, 128, sk.SK_BF16),
              (300, 48, 80, 3, 16, sk.SK_F32)):
        both = sk.sk_linear_workspace_bytes(sk.SK_OP_BWD, *a)
        parts = (sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_INPUT, *a) +
                 sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT, *a))
        assert both >= parts            # room for the two gradients' buffers side by side
        assert f(P, P, P, P, P, P, None, *a, P, both - 1) == sk.SK_ERR_WORKSPACE


def test_noalloc_entry_rejects_before_any_hip_call():
    f = sk.sk_linear_bwd_weight_noalloc
    assert f(None, P, P, P, P, *ARGS) == sk.SK_ERR_INVALID_ARG
    assert f(P, P, P, P, P + 4, *ARGS) == sk.SK_ERR_INVALID_ARG
    assert f(P, P, P, P, None, 64, 64, 60, 1, 16, sk.SK_BF16) == sk.SK_ERR_UNSUPPORTED
    # a workspace larger than the fixed scratch array: refused, nothing enqueued
    big = (16384, 4096, 11008, 8, 256, sk.SK_BF16)
    assert sk.sk_linear_workspace_bytes(sk.SK_OP_BWD_WEIGHT, *big) > sk.SK_NOALLOC_SCRATCH_BYTES
    assert f(P, P, P, P, None, *big) == sk.SK_ERR_WORKSPACE
    hdr = open(os.path.join(ROOT, "include", "sk.h")).read()
    assert re.search(r"#define SK_NOALLOC_SCRATCH_BYTES \(32u << 20\)", hdr)
    assert sk.SK_NOALLOC_SCRATCH_BYTES == 32 << 20
