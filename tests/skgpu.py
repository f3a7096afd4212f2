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


def abs_err_scaled(got: np.ndarray, want: np.ndarray) -> float:
    """A second figure beside rel_err: max_i |g_i - o_i| / max_i |o_i| over the whole tensor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if not np.all(np.isfinite(got)):
        return float("inf")
    top = float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want))) / (top if top > 0.0 else 1.0)


def errors_by_row_blocks(got_dev: torch.Tensor, want: np.ndarray, block: int = 1024):
    """(rel_err, abs_err_scaled) of a large device tensor against the oracle's array, brought
    back and compared a block of rows at a time so that only one block is held in fp64 twice."""
    assert tuple(got_dev.shape) == want.shape, (tuple(got_dev.shape), want.shape)
    top = float(np.max(np.abs(want)))
    worst_rel, worst_abs = 0.0, 0.0
    for r0 in range(0, want.shape[0], block):
        g = to_f64(got_dev[r0:r0 + block])
        w = want[r0:r0 + block]
        worst_rel = max(worst_rel, rel_err(g, w))
        if not np.all(np.isfinite(g)):
            return float("inf"), float("inf")
        worst_abs = max(worst_abs, float(np.max(np.abs(g - w))))
    return worst_rel, worst_abs / (top if top > 0.0 else 1.0)
