"""Device-side plumbing for libsk: puts a workload's tensors into HBM (PyTorch is
used for allocation and streams only) and wires up the three C-ABI calls."""
from __future__ import annotations

import numpy as np
import torch

from . import workloads as W


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Storage-form array -> device tensor (bf16 arrives as uint16 bit patterns)."""
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class DeviceLayer:
    """A workload resident on the GPU, with the three libsk calls wired up."""

    def __init__(self, tensors: W.Tensors, libsk, poison=True):
        self.t = tensors
        self.w = tensors.workload
        self.sk = libsk
        w = self.w
        self.dt = libsk.DTYPES[w.dtype]
        self.tdtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.x = to_dev(tensors.stored["x"], w.dtype)
        self.dY = to_dev(tensors.stored["dY"], w.dtype)
        self.S_cat = to_dev(tensors.S_cat(), w.dtype)
        self.U_cat = to_dev(tensors.U_cat(), w.dtype)
        self.b = to_dev(tensors.stored["b"], w.dtype) if "b" in tensors.stored else None
        fill = float("nan") if poison else 0.0
        self.y = torch.full((w.tokens, w.d_out), fill, dtype=self.tdtype, device="cuda")
        self.dX = torch.full((w.tokens, w.d_in), fill, dtype=self.tdtype, device="cuda")
        self.dU = torch.full((w.R, w.d_out), fill, dtype=torch.float32, device="cuda")
        self.db = torch.full((w.d_out,), fill, dtype=torch.float32, device="cuda")
        self.args = (w.tokens, w.d_in, w.d_out, w.l, w.k, self.dt)
        need = max(libsk.sk_linear_workspace_bytes(op, *self.args) for op in (0, 1, 2, 4))
        assert need != 2 ** 64 - 1
        self.ws_bytes = need
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def bwd(self, stream=None, with_db=True):
        """Both gradients in one call (sk_linear_bwd)."""
        return self.sk.sk_linear_bwd(self.x, self.dY, self.S_cat, self.U_cat, self.dX, self.dU,
                                     self.db if with_db else None, *self.args,
                                     self.ws, self.ws_bytes, stream)

    def fwd(self, stream=None):
        return self.sk.sk_linear_fwd(self.x, self.S_cat, self.U_cat, self.b, self.y, *self.args,
                                     self.ws, self.ws_bytes, stream)

    def bwd_input(self, stream=None):
        return self.sk.sk_linear_bwd_input(self.dY, self.S_cat, self.U_cat, self.dX, *self.args,
                                           self.ws, self.ws_bytes, stream)

    def bwd_weight(self, stream=None, with_db=True):
        return self.sk.sk_linear_bwd_weight(self.x, self.S_cat, self.dY, self.dU,
                                            self.db if with_db else None, *self.args,
                                            self.ws, self.ws_bytes, stream)

    def run_all(self):
        for st in (self.fwd(), self.bwd_input(), self.bwd_weight()):
            self.sk.check(st)
        torch.cuda.synchronize()


class TwoSidedDeviceLayer(DeviceLayer):
    """The two-sided reading of the layer (workloads.generate_two_sided: ``w.l`` terms per
    side) resident on the GPU: the three calls run on the concatenated stage matrices with
    2 l terms, and ``bwd_weight_first`` computes the gradient of the learned first-stage
    columns (the second half of A_cat) into ``dA`` [in, l*k]."""

    def __init__(self, tensors: W.Tensors, libsk, poison=True):
        w = tensors.workload
        self.t, self.w, self.sk = tensors, w, libsk
        self.dt = libsk.DTYPES[w.dtype]
        self.tdtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.x = to_dev(tensors.stored["x"], w.dtype)
        self.dY = to_dev(tensors.stored["dY"], w.dtype)
        self.S_cat = to_dev(tensors.stored["A_cat"], w.dtype)
        self.U_cat = to_dev(tensors.stored["B_cat"], w.dtype)
        self.b = to_dev(tensors.stored["b"], w.dtype)
        fill = float("nan") if poison else 0.0
        R, self.half = 2 * w.R, w.R
        self.y = torch.full((w.tokens, w.d_out), fill, dtype=self.tdtype, device="cuda")
        self.dX = torch.full((w.tokens, w.d_in), fill, dtype=self.tdtype, device="cuda")
        self.dU = torch.full((R, w.d_out), fill, dtype=torch.float32, device="cuda")
        self.db = torch.full((w.d_out,), fill, dtype=torch.float32, device="cuda")
        self.dA = torch.full((w.d_in, self.half), fill, dtype=torch.float32, device="cuda")
        self.args = (w.tokens, w.d_in, w.d_out, 2 * w.l, w.k, self.dt)
        need = max(libsk.sk_linear_workspace_bytes(op, *self.args) for op in (0, 1, 2, 3))
        assert need != 2 ** 64 - 1
        self.ws_bytes = need
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def bwd_weight_first(self, stream=None):
        return self.sk.sk_linear_bwd_weight_first(
            self.x, self.U_cat, self.dY, self.dA, *self.args[:5], self.half, self.half, self.dt,
            self.ws, self.ws_bytes, stream)

    def run_all(self):
        for st in (self.fwd(), self.bwd_input(), self.bwd_weight(), self.bwd_weight_first()):
            self.sk.check(st)
        torch.cuda.synchronize()
