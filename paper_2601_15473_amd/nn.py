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

import math

import torch

from . import libsk as sk

_DTYPES = {torch.float32: sk.SK_F32, torch.bfloat16: sk.SK_BF16}
_workspaces: dict = {}


def _workspace(device: torch.device, stream: int, nbytes: int) -> torch.Tensor:
    """One scratch buffer per (device, stream): calls on a stream run in order, so they
    can share it; it only ever grows."""
    key = (device.index, stream)
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


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
