"""PyTorch surface of the sketched linear layer: ``SKLinear(in_features,
out_features, num_terms, low_rank)`` as a drop-in for ``torch.nn.Linear`` (the
paper's "Tool Usage" section: the layer averages ``num_terms`` sketched products
whose sketches have rank ``low_rank``), with autograd support.

Everything that computes runs in libsk's HIP kernels: ``forward`` calls
``sk_linear_fwd``; ``backward`` calls ``sk_linear_bwd`` (both gradients in one
call) or, when only one of them is wanted, ``sk_linear_bwd_input`` or
``sk_linear_bwd_weight``; the factor gradient recomputes x.S rather than keeping
it from the forward pass.  PyTorch provides the tensors, the stream and the autograd graph.
There is no CPU path: tensors that are not on a GPU raise.

    y = (1/l) * sum_i (x . S_i) . U_i + b        S_i fixed random, U_i and b learned
"""
from __future__ import annotations

import collections
import math

import torch

from . import libsk as sk

_DTYPES = {torch.float32: sk.SK_F32, torch.bfloat16: sk.SK_BF16}
_workspaces: "collections.OrderedDict" = collections.OrderedDict()
_MAX_WORKSPACES = 8


def _workspace(device: torch.device, stream: int, nbytes: int) -> torch.Tensor:
    """One scratch buffer per (device, stream): calls on a stream run in order, so they can
    share it.  A buffer grows to the largest request seen on its stream; at most
    ``_MAX_WORKSPACES`` streams keep one (least recently used dropped first: torch's caching
    allocator keeps a dropped buffer alive until the work queued on it is done), and
    ``release_workspaces()`` drops them all."""
    key = (device.index, stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    _workspaces.move_to_end(key)
    while len(_workspaces) > _MAX_WORKSPACES:
        _workspaces.popitem(last=False)
    return ws


def release_workspaces() -> None:
    """Give the layers' scratch buffers back to the allocator (they are re-created on demand)."""
    _workspaces.clear()


def _check(x: torch.Tensor, name: str, dtype: torch.dtype):
    if not x.is_cuda:
        raise RuntimeError(f"SKLinear: {name} is on {x.device}; libsk runs on the GPU only "
                           "(there is no CPU implementation)")
    if x.dtype != dtype:
        raise TypeError(f"SKLinear: {name} has dtype {x.dtype}, the layer's is {dtype}")


class SKLinearFunction(torch.autograd.Function):
    """y = sklinear(x, S_cat, U_cat, bias); S_cat [in, l*k] gets no gradient (fixed sketch)."""

    @staticmethod
    def forward(ctx, x, S_cat, U_cat, bias, l, k):
        dtype = S_cat.dtype
        if dtype not in _DTYPES:
            raise TypeError(f"SKLinear: dtype {dtype} is not supported (float32 or bfloat16)")
        d_in, R = S_cat.shape
        d_out = U_cat.shape[1]
        if R != l * k or U_cat.shape[0] != R or x.shape[-1] != d_in:
            raise ValueError("SKLinear: shapes do not match (x [..., in], S_cat [in, l*k], U_cat [l*k, out])")
        for t, n in ((x, "x"), (S_cat, "S_cat"), (U_cat, "U_cat")) + (((bias, "bias"),) if bias is not None else ()):
            _check(t, n, dtype)
        x2 = x.reshape(-1, d_in).contiguous()
        S_cat, U_cat = S_cat.contiguous(), U_cat.contiguous()
        bias_c = bias.contiguous() if bias is not None else None
        tokens = x2.shape[0]
        y = torch.empty((tokens, d_out), dtype=dtype, device=x.device)
        args = (tokens, d_in, d_out, l, k, _DTYPES[dtype])
        with torch.cuda.device(x.device):
            stream = torch.cuda.current_stream().cuda_stream
            need = sk.sk_linear_workspace_bytes(sk.SK_OP_FWD, *args)
            if need == 2 ** 64 - 1:
                raise sk.SkError(sk.SK_ERR_UNSUPPORTED)
            ws = _workspace(x.device, stream, need)
            sk.check(sk.sk_linear_fwd(x2, S_cat, U_cat, bias_c, y, *args, ws, ws.numel(), stream))
        ctx.save_for_backward(x2, S_cat, U_cat)
        ctx.args = args
        ctx.x_shape = x.shape
        ctx.has_bias = bias is not None
        return y.reshape(*x.shape[:-1], d_out)

    @staticmethod
    def backward(ctx, dY):
        x2, S_cat, U_cat = ctx.saved_tensors
        tokens, d_in, d_out, l, k, dt = ctx.args
        dtype = S_cat.dtype
        dY2 = dY.reshape(-1, d_out).to(dtype).contiguous()
        need_dx, _, need_du, need_db = ctx.needs_input_grad[:4]
        dX = dU = db = None
        with torch.cuda.device(dY.device):
            stream = torch.cuda.current_stream().cuda_stream
            want_w = need_du or (need_db and ctx.has_bias)
            need = max(sk.sk_linear_workspace_bytes(op, *ctx.args)
                       for op in (sk.SK_OP_BWD_INPUT, sk.SK_OP_BWD_WEIGHT, sk.SK_OP_BWD))
            ws = _workspace(dY.device, stream, need)
            if need_dx:
                dX = torch.empty((tokens, d_in), dtype=dtype, device=dY.device)
            if want_w:
                dU32 = torch.empty((l * k, d_out), dtype=torch.float32, device=dY.device)
                db32 = torch.empty((d_out,), dtype=torch.float32, device=dY.device) if ctx.has_bias else None
            if need_dx and want_w:      # both gradients from one call (its kernels share launches)
                sk.check(sk.sk_linear_bwd(x2, dY2, S_cat, U_cat, dX, dU32, db32, *ctx.args,
                                          ws, ws.numel(), stream))
            elif need_dx:
                sk.check(sk.sk_linear_bwd_input(dY2, S_cat, U_cat, dX, *ctx.args, ws, ws.numel(), stream))
            elif want_w:
                sk.check(sk.sk_linear_bwd_weight(x2, S_cat, dY2, dU32, db32, *ctx.args, ws, ws.numel(), stream))
            if need_dx:
                dX = dX.reshape(ctx.x_shape)
            if want_w:
                dU = dU32.to(dtype) if need_du else None
                db = db32.to(dtype) if (need_db and ctx.has_bias) else None
        return dX, None, dU, db, None, None


def sklinear(x, S_cat, U_cat, bias, num_terms: int, low_rank: int):
    """Functional form; see SKLinearFunction."""
    return SKLinearFunction.apply(x, S_cat, U_cat, bias, num_terms, low_rank)


class SKLinear(torch.nn.Module):
    """Sketched drop-in for ``torch.nn.Linear`` (the paper's SKLinear).

    ``S_cat [in, l*k]`` holds the l fixed Gaussian sketches side by side (entries
    N(0, 1/k), so that E[S_i S_i^T] = I) and is a buffer; ``U_cat [l*k, out]`` holds
    the learned factors stacked (term i in rows i*k .. i*k+k-1) and is a parameter,
    as is ``bias``.  All sizes must be multiples of 16.
    """

    def __init__(self, in_features: int, out_features: int, num_terms: int = 1, low_rank: int = 16,
                 bias: bool = True, dtype: torch.dtype = torch.bfloat16, device="cuda", seed: int | None = None):
        super().__init__()
        if dtype not in _DTYPES:
            raise TypeError(f"SKLinear: dtype {dtype} is not supported (float32 or bfloat16)")
        device = torch.device(device)
        if device.type != "cuda":
            raise RuntimeError("SKLinear: libsk runs on the GPU only (there is no CPU implementation)")
        self.in_features, self.out_features = in_features, out_features
        self.num_terms, self.low_rank = num_terms, low_rank
        R = num_terms * low_rank
        g = torch.Generator(device="cpu")
        if seed is not None:
            g.manual_seed(seed)
        else:
            g.seed()
        S = torch.randn(in_features, R, generator=g) / math.sqrt(low_rank)
        # factors of a dense layer initialised the way nn.Linear is: U_i = S_i^T . W^T
        bound = 1.0 / math.sqrt(in_features)
        W = (torch.rand(out_features, in_features, generator=g) * 2 - 1) * bound
        self.register_buffer("S_cat", S.to(dtype).to(device))
        self.U_cat = torch.nn.Parameter((self.S_cat.float().t() @ W.t().to(device)).to(dtype))
        if bias:
            b = (torch.rand(out_features, generator=g) * 2 - 1) * bound
            self.bias = torch.nn.Parameter(b.to(dtype).to(device))
        else:
            self.register_parameter("bias", None)

    @classmethod
    def from_linear(cls, linear: torch.nn.Linear, num_terms: int, low_rank: int,
                    dtype: torch.dtype = torch.bfloat16, seed: int | None = None) -> "SKLinear":
        """Sketched layer that keeps a trained dense layer's weights (the tuner's
        ``copy_weights`` option): U_i = S_i^T . W^T, so that the layer's expectation over
        the sketches is the dense layer."""
        m = cls(linear.in_features, linear.out_features, num_terms, low_rank,
                bias=linear.bias is not None, dtype=dtype, device=linear.weight.device, seed=seed)
        with torch.no_grad():
            m.U_cat.copy_((m.S_cat.float().t() @ linear.weight.detach().float().t()).to(dtype))
            if linear.bias is not None:
                m.bias.copy_(linear.bias.detach().to(dtype))
        return m

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return SKLinearFunction.apply(x, self.S_cat, self.U_cat, self.bias, self.num_terms, self.low_rank)

    def extra_repr(self) -> str:
        return (f"in_features={self.in_features}, out_features={self.out_features}, "
                f"num_terms={self.num_terms}, low_rank={self.low_rank}, bias={self.bias is not None}")


class SKLinearTwoSidedFunction(torch.autograd.Function):
    """The two-sided reading of the layer (2 l terms: l sketch the input side, l the output
    side; see include/sk.h, sk_linear_bwd_weight_first):

        y = 1/(2l) * sum_i [ (x . S1_i) . U1_i + (x . U2_i) . S2_i^T ] + b

    Arguments: S1_cat [in, l*k] and S2T_cat [l*k, out] fixed, U1_cat [l*k, out] and U2_cat
    [in, l*k] learned.  The layer is the one-sided chain on [S1 | U2] and [U1 ; S2^T] with 2 l
    terms; ``stage`` may carry those two concatenations ready made (the module caches them
    until a learned factor changes), otherwise they are copied together here; everything else
    runs in libsk."""

    @staticmethod
    def forward(ctx, x, S1_cat, U1_cat, U2_cat, S2T_cat, bias, l, k, stage=None):
        dtype = S1_cat.dtype
        if dtype not in _DTYPES:
            raise TypeError(f"SKLinear: dtype {dtype} is not supported (float32 or bfloat16)")
        for t, n in ((x, "x"), (S1_cat, "S1_cat"), (U1_cat, "U1_cat"), (U2_cat, "U2_cat"), (S2T_cat, "S2T_cat")):
            _check(t, n, dtype)
        d_in, half = S1_cat.shape
        d_out = U1_cat.shape[1]
        if half != l * k or U1_cat.shape[0] != half or U2_cat.shape != (d_in, half) or \
                S2T_cat.shape != (half, d_out) or x.shape[-1] != d_in:
            raise ValueError("SKLinear (two-sided): shapes do not match")
        if stage is not None:
            A_cat, B_cat = stage
        else:
            A_cat = torch.cat([S1_cat, U2_cat], dim=1).contiguous()
            B_cat = torch.cat([U1_cat, S2T_cat], dim=0).contiguous()
        x2 = x.reshape(-1, d_in).contiguous()
        bias_c = bias.contiguous() if bias is not None else None
        tokens = x2.shape[0]
        y = torch.empty((tokens, d_out), dtype=dtype, device=x.device)
        args = (tokens, d_in, d_out, 2 * l, k, _DTYPES[dtype])
        with torch.cuda.device(x.device):
            stream = torch.cuda.current_stream().cuda_stream
            need = sk.sk_linear_workspace_bytes(sk.SK_OP_FWD, *args)
            if need == 2 ** 64 - 1:
                raise sk.SkError(sk.SK_ERR_UNSUPPORTED)
            ws = _workspace(x.device, stream, need)
            sk.check(sk.sk_linear_fwd(x2, A_cat, B_cat, bias_c, y, *args, ws, ws.numel(), stream))
        ctx.save_for_backward(x2, A_cat, B_cat)
        ctx.args, ctx.x_shape, ctx.has_bias, ctx.half = args, x.shape, bias is not None, half
        return y.reshape(*x.shape[:-1], d_out)

    @staticmethod
    def backward(ctx, dY):
        x2, A_cat, B_cat = ctx.saved_tensors
        tokens, d_in, d_out, l2, k, dt = ctx.args
        dtype, half = A_cat.dtype, ctx.half
        dY2 = dY.reshape(-1, d_out).to(dtype).contiguous()
        dev = dY.device
        with torch.cuda.device(dev):
            stream = torch.cuda.current_stream().cuda_stream
            need = max(sk.sk_linear_workspace_bytes(op, *ctx.args)
                       for op in (sk.SK_OP_BWD, sk.SK_OP_BWD_WEIGHT_FIRST))
            ws = _workspace(dev, stream, need)
            dX = torch.empty((tokens, d_in), dtype=dtype, device=dev)
            dB = torch.empty((2 * half, d_out), dtype=torch.float32, device=dev)
            db = torch.empty((d_out,), dtype=torch.float32, device=dev) if ctx.has_bias else None
            dA = torch.empty((d_in, half), dtype=torch.float32, device=dev)
            sk.check(sk.sk_linear_bwd(x2, dY2, A_cat, B_cat, dX, dB, db, *ctx.args, ws, ws.numel(), stream))
            sk.check(sk.sk_linear_bwd_weight_first(x2, B_cat, dY2, dA, tokens, d_in, d_out, l2, k,
                                                   half, half, dt, ws, ws.numel(), stream))
        # the rows of dB below `half` belong to S2^T: gradients of fixed numbers, dropped
        return (dX.reshape(ctx.x_shape), None, dB[:half].to(dtype), dA.to(dtype), None,
                db.to(dtype) if db is not None else None, None, None, None)


class SKLinearTwoSided(torch.nn.Module):
    """``SKLinear`` in its two-sided reading: ``num_terms`` terms per side.  Initialised from
    a dense layer's weights the way ``SKLinear`` is: U1_i = S1_i^T W^T, U2_i = W^T S2_i."""

    def __init__(self, in_features: int, out_features: int, num_terms: int = 1, low_rank: int = 16,
                 bias: bool = True, dtype: torch.dtype = torch.bfloat16, device="cuda", seed: int | None = None):
        super().__init__()
        if dtype not in _DTYPES:
            raise TypeError(f"SKLinear: dtype {dtype} is not supported (float32 or bfloat16)")
        device = torch.device(device)
        if device.type != "cuda":
            raise RuntimeError("SKLinear: libsk runs on the GPU only (there is no CPU implementation)")
        self.in_features, self.out_features = in_features, out_features
        self.num_terms, self.low_rank = num_terms, low_rank
        half = num_terms * low_rank
        g = torch.Generator(device="cpu")
        if seed is not None:
            g.manual_seed(seed)
        else:
            g.seed()
        S1 = (torch.randn(in_features, half, generator=g) / math.sqrt(low_rank)).to(dtype).to(device)
        S2T = (torch.randn(half, out_features, generator=g) / math.sqrt(low_rank)).to(dtype).to(device)
        bound = 1.0 / math.sqrt(in_features)
        W = ((torch.rand(out_features, in_features, generator=g) * 2 - 1) * bound).to(device)
        self.register_buffer("S1_cat", S1)
        self.register_buffer("S2T_cat", S2T)
        self.U1_cat = torch.nn.Parameter((S1.float().t() @ W.t()).to(dtype))       # [l*k, out]
        self.U2_cat = torch.nn.Parameter((W.t() @ S2T.float().t()).to(dtype))      # [in, l*k]
        self._stage, self._stage_key = None, None
        if bias:
            b = (torch.rand(out_features, generator=g) * 2 - 1) * bound
            self.bias = torch.nn.Parameter(b.to(dtype).to(device))
        else:
            self.register_parameter("bias", None)

    def _stage_matrices(self):
        """[S1 | U2] and [U1 ; S2^T], rebuilt only when a learned factor (or a buffer) has been
        written since the cached copies were made -- tensors count their in-place writes, which
        is how optimizers update parameters.  Stale copies are replaced, never overwritten: a
        backward pass that is still to come holds the ones its forward pass used."""
        parts = (self.S1_cat, self.U2_cat, self.U1_cat, self.S2T_cat)
        key = tuple((t.data_ptr(), t._version, t.dtype) for t in parts)
        if self._stage_key != key:
            with torch.no_grad():
                self._stage = (torch.cat([self.S1_cat, self.U2_cat], dim=1).contiguous(),
                               torch.cat([self.U1_cat, self.S2T_cat], dim=0).contiguous())
            self._stage_key = key
        return self._stage

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return SKLinearTwoSidedFunction.apply(x, self.S1_cat, self.U1_cat, self.U2_cat, self.S2T_cat,
                                              self.bias, self.num_terms, self.low_rank, self._stage_matrices())

    def extra_repr(self) -> str:
        return (f"in_features={self.in_features}, out_features={self.out_features}, "
                f"num_terms={self.num_terms} per side, low_rank={self.low_rank}, bias={self.bias is not None}")
