"""Helpers of the GPU parity tests: bring results back as fp64 and measure the
error against the oracle.  (Not a test module.)"""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_15473_amd.device import DeviceLayer, to_dev  # noqa: F401

TOL = {"f32": 1e-4, "bf16": 2e-2}   # the stated parity tolerances


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |g_i - o_i| / max(|o_i|, rms of the row o_i sits in).

    Element-wise relative error is unbounded where the exact value crosses
    zero, so each element is judged at the larger of its own magnitude and the
    rms of its row (token row for y/dX, R-row for dU, whole vector for 1-D)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if not np.all(np.isfinite(got)):
        return float("inf")
    w2 = want.reshape(1, -1) if want.ndim == 1 else want.reshape(want.shape[0], -1)
    g2 = got.reshape(w2.shape)
    rms = np.sqrt(np.mean(w2 * w2, axis=1, keepdims=True))
    denom = np.maximum(np.abs(w2), rms)
    denom = np.where(denom == 0.0, 1.0, denom)
    return float(np.max(np.abs(g2 - w2) / denom))
