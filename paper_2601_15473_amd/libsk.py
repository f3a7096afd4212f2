"""ctypes binding of libsk.so: the entry points of include/sk.h under the same
names.  Argument marshalling only -- every step of the computation runs in the
library's HIP kernels.  There is no CPU fallback: if the library has not been
built (``python -m paper_2601_15473_amd.build``) importing this module fails.

Pointer arguments may be given as integers (device addresses), objects with a
``data_ptr()`` method (torch tensors) or None.  ``stream`` may be an integer
handle, an object with a ``cuda_stream`` attribute (torch.cuda.Stream) or None
for the default stream.
"""
from __future__ import annotations

import ctypes
import os

# Load order matters: PyTorch ships its own copy of the HIP runtime under the same soname
# as the system's, and a process can hold only one of them.  The runtime that owns the
# tensors' memory and streams must be the one libsk's launches go through, so torch (when
# it is installed) is imported before libsk.so pulls in a runtime of its own.
try:
    import torch  # noqa: F401
except ImportError:   # plain-pointer callers without PyTorch
    pass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libsk.so")

SK_OK, SK_ERR_INVALID_ARG, SK_ERR_UNSUPPORTED, SK_ERR_WORKSPACE, SK_ERR_HIP = range(5)
SK_F32, SK_BF16 = 0, 1
SK_NOALLOC_SCRATCH_BYTES = 32 << 20   # fixed scratch of sk_linear_bwd_weight_noalloc
SK_OP_FWD, SK_OP_BWD_INPUT, SK_OP_BWD_WEIGHT, SK_OP_BWD_WEIGHT_FIRST, SK_OP_BWD = 0, 1, 2, 3, 4
DTYPES = {"f32": SK_F32, "bf16": SK_BF16}

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2601_15473_amd.build` "
        "(there is no fallback implementation)")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _i32, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
_tail = [_i64, _i64, _i64, _i32, _i32, ctypes.c_int, _vp, _sz, _vp]

_lib.sk_linear_fwd.restype = ctypes.c_int
_lib.sk_linear_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp] + _tail
_lib.sk_linear_bwd_input.restype = ctypes.c_int
_lib.sk_linear_bwd_input.argtypes = [_vp, _vp, _vp, _vp] + _tail
_lib.sk_linear_bwd_weight.restype = ctypes.c_int
_lib.sk_linear_bwd_weight.argtypes = [_vp, _vp, _vp, _vp, _vp] + _tail
_lib.sk_linear_bwd_weight_noalloc.restype = ctypes.c_int
_lib.sk_linear_bwd_weight_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i32, _i32,
                                              ctypes.c_int, _vp]
_lib.sk_linear_bwd.restype = ctypes.c_int
_lib.sk_linear_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp] + _tail
_lib.sk_linear_bwd_weight_first.restype = ctypes.c_int
_lib.sk_linear_bwd_weight_first.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _i32, _i32, _i64, _i64,
                                            ctypes.c_int, _vp, _sz, _vp]
_lib.sk_linear_workspace_bytes.restype = _sz
_lib.sk_linear_workspace_bytes.argtypes = [ctypes.c_int, _i64, _i64, _i64, _i32, _i32, ctypes.c_int]
_lib.sk_status_string.restype = ctypes.c_char_p
_lib.sk_status_string.argtypes = [ctypes.c_int]
_lib.sk_last_hip_error.restype = ctypes.c_char_p
_lib.sk_last_hip_error.argtypes = []
_lib.sk_set_plan.restype = ctypes.c_int
_lib.sk_set_plan.argtypes = [ctypes.c_int]

# ---- testing / tuning / measurement aids (include/sk_debug.h) ----
(SK_TUNE_TILE, SK_TUNE_WTILE, SK_TUNE_WSPLITS, SK_TUNE_BM, SK_TUNE_SLICES, SK_TUNE_STILE, SK_TUNE_SSPLITS,
 SK_TUNE_NARROW_BWD) = range(8)


class TraceAccess(ctypes.Structure):
    _fields_ = [("address", ctypes.c_uint64), ("bytes", ctypes.c_uint64),
                ("write", ctypes.c_int32), ("launch", ctypes.c_int32)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 120), ("ms", ctypes.c_float), ("groups", ctypes.c_int32),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


_lib.sk_set_tuning.restype = ctypes.c_int32
_lib.sk_set_tuning.argtypes = [ctypes.c_int, ctypes.c_int32]
_lib.sk_trace_begin.restype = None
_lib.sk_trace_begin.argtypes = []
_lib.sk_trace_end.restype = ctypes.c_int64
_lib.sk_trace_end.argtypes = [ctypes.POINTER(TraceAccess), ctypes.c_int64, ctypes.POINTER(ctypes.c_int32)]
_lib.sk_profile_begin.restype = ctypes.c_int32
_lib.sk_profile_begin.argtypes = [ctypes.c_int32]
_lib.sk_profile_end.restype = ctypes.c_int32
_lib.sk_profile_end.argtypes = [ctypes.POINTER(KernelTime), ctypes.c_int32]

DEBUG_EXPORTS = ("sk_set_tuning", "sk_trace_begin", "sk_trace_end", "sk_profile_begin", "sk_profile_end")

EXPORTS = ("sk_linear_fwd", "sk_linear_bwd_input", "sk_linear_bwd_weight", "sk_linear_bwd",
           "sk_linear_bwd_weight_first", "sk_linear_bwd_weight_noalloc",
           "sk_linear_workspace_bytes", "sk_status_string", "sk_last_hip_error", "sk_set_plan")


class SkError(RuntimeError):
    def __init__(self, status):
        self.status = status
        msg = sk_status_string(status)
        if status == SK_ERR_HIP:
            msg += " -- " + sk_last_hip_error()
        super().__init__(msg)


def _ptr(a):
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.data_ptr()


def _stream(s):
    if s is None or isinstance(s, int):
        return s
    return s.cuda_stream


def sk_linear_fwd(x, S_cat, U_cat, bias, y, tokens, d_in, d_out, l, k, dtype,
                  workspace, workspace_bytes, stream=None):
    return _lib.sk_linear_fwd(_ptr(x), _ptr(S_cat), _ptr(U_cat), _ptr(bias), _ptr(y),
                              tokens, d_in, d_out, l, k, dtype,
                              _ptr(workspace), workspace_bytes, _stream(stream))


def sk_linear_bwd_input(dY, S_cat, U_cat, dX, tokens, d_in, d_out, l, k, dtype,
                        workspace, workspace_bytes, stream=None):
    return _lib.sk_linear_bwd_input(_ptr(dY), _ptr(S_cat), _ptr(U_cat), _ptr(dX),
                                    tokens, d_in, d_out, l, k, dtype,
                                    _ptr(workspace), workspace_bytes, _stream(stream))


def sk_linear_bwd_weight(x, S_cat, dY, dU_cat, dbias, tokens, d_in, d_out, l, k, dtype,
                         workspace, workspace_bytes, stream=None):
    return _lib.sk_linear_bwd_weight(_ptr(x), _ptr(S_cat), _ptr(dY), _ptr(dU_cat), _ptr(dbias),
                                     tokens, d_in, d_out, l, k, dtype,
                                     _ptr(workspace), workspace_bytes, _stream(stream))


def sk_linear_bwd_weight_noalloc(x, S_cat, dY, dU_cat, dbias, tokens, d_in, d_out, l, k, dtype,
                                 stream=None):
    return _lib.sk_linear_bwd_weight_noalloc(_ptr(x), _ptr(S_cat), _ptr(dY), _ptr(dU_cat), _ptr(dbias),
                                             tokens, d_in, d_out, l, k, dtype, _stream(stream))


def sk_linear_bwd(x, dY, S_cat, U_cat, dX, dU_cat, dbias, tokens, d_in, d_out, l, k, dtype,
                  workspace, workspace_bytes, stream=None):
    return _lib.sk_linear_bwd(_ptr(x), _ptr(dY), _ptr(S_cat), _ptr(U_cat), _ptr(dX), _ptr(dU_cat),
                              _ptr(dbias), tokens, d_in, d_out, l, k, dtype,
                              _ptr(workspace), workspace_bytes, _stream(stream))


def sk_linear_bwd_weight_first(x, U_cat, dY, dA, tokens, d_in, d_out, l, k, col_begin, col_count, dtype,
                               workspace, workspace_bytes, stream=None):
    return _lib.sk_linear_bwd_weight_first(_ptr(x), _ptr(U_cat), _ptr(dY), _ptr(dA),
                                           tokens, d_in, d_out, l, k, col_begin, col_count, dtype,
                                           _ptr(workspace), workspace_bytes, _stream(stream))


def sk_linear_workspace_bytes(op, tokens, d_in, d_out, l, k, dtype):
    return _lib.sk_linear_workspace_bytes(op, tokens, d_in, d_out, l, k, dtype)


def sk_status_string(status):
    return _lib.sk_status_string(status).decode()


def sk_last_hip_error():
    return _lib.sk_last_hip_error().decode()


def sk_set_plan(plan):
    return _lib.sk_set_plan(plan)


def sk_set_tuning(knob, value):
    """Force a plan parameter (value < 0: automatic again); returns the previous value."""
    return _lib.sk_set_tuning(knob, value)


def sk_trace_begin():
    _lib.sk_trace_begin()


_trace_buf = (TraceAccess * 256)()


def sk_trace_end():
    """-> (list of (address, bytes, write, launch), number of launches)."""
    launches = ctypes.c_int32(0)
    n = _lib.sk_trace_end(_trace_buf, len(_trace_buf), ctypes.byref(launches))
    if n > len(_trace_buf):
        raise RuntimeError(f"launch trace holds {n} records, buffer {len(_trace_buf)}")
    return [(a.address, a.bytes, a.write, a.launch) for a in _trace_buf[:n]], launches.value


def sk_profile_begin(max_kernels):
    rc = _lib.sk_profile_begin(max_kernels)
    if rc != 0:
        raise RuntimeError(f"sk_profile_begin failed ({rc})")


def sk_profile_end(max_kernels):
    """-> list of (kernel name, ms, work-groups, flops, bytes), one per launch, in launch order."""
    buf = (KernelTime * max_kernels)()
    n = _lib.sk_profile_end(buf, max_kernels)
    if n < 0:
        raise RuntimeError(f"sk_profile_end failed ({n})")
    return [(k.name.decode(), float(k.ms), int(k.groups), float(k.flops), float(k.bytes))
            for k in buf[:min(n, max_kernels)]]


def check(status):
    """Raise SkError unless ``status`` is SK_OK."""
    if status != SK_OK:
        raise SkError(status)
