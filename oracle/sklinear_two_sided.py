"""Plain fp64 oracle of the TWO-SIDED reading of the sketched linear layer.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

Why a second reading: the paper's size rule (Sec. 4.1) counts a sketched layer as
2 l k (d_in + d_out) numbers, twice what the one-sided layer of ``sklinear.py``
stores.  The count fits a layer with 2 l terms: l that sketch the input side
(fixed S1_i, in x k, then learned U1_i, k x out -- the one-sided layer) and l that
sketch the output side (learned U2_i, in x k, then fixed S2_i^T, k x out), all
averaged.  The paper prints no formula, so this is a reading of that count, not
a quotation:

    y = 1/(2l) * sum_i [ (x . S1_i) . U1_i  +  (x . U2_i) . S2_i^T ] + b      (T1)

Gradients are the exact derivatives of L = sum(dY * y); S1_i and S2_i are fixed:

    dX    = 1/(2l) * sum_i [ (dY . U1_i^T) . S1_i^T + (dY . S2_i) . U2_i^T ]   (T2)
    dU1_i = 1/(2l) * (x . S1_i)^T . dY                                         (T3)
    dU2_i = 1/(2l) * x^T . (dY . S2_i)                                         (T4)
    db    = sum over tokens of dY                                              (T5)

One term at a time, one library matmul per product, fp64 throughout, nothing
concatenated.  Arrays: x [T, in], S1 [l, in, k], U1 [l, k, out], U2 [l, in, k],
S2 [l, out, k], b [out] or None.

Pinned (tests/test_oracle_pins.py) by: central finite differences in x, U1, U2 and
b (L is linear in each), the dense special case (k = in = out, S1 = S2 = I gives
x . (U1 + U2) / 2 + b), equality with the one-sided oracle run on the concatenated
stage matrices [S1 | U2] and [U1 ; S2^T] with 2 l terms (which also pins the layout
the GPU path uses), the stored-number count against the paper's size rule, and the
expectation of the estimator over Gaussian sketches.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _check(x_cols, out_cols, S1, U1, U2, S2):
    S1, U1, U2, S2 = _f64(S1), _f64(U1), _f64(U2), _f64(S2)
    l, d_in, k = S1.shape
    if U1.shape[:2] != (l, k) or U2.shape != (l, d_in, k) or S2.shape[0] != l or S2.shape[2] != k:
        raise ValueError("expected S1 [l,in,k], U1 [l,k,out], U2 [l,in,k], S2 [l,out,k]")
    if U1.shape[2] != S2.shape[1]:
        raise ValueError("U1 and S2 disagree on the output dimension")
    if x_cols is not None and x_cols != d_in:
        raise ValueError("feature dimension of x does not match the sketches")
    if out_cols is not None and out_cols != U1.shape[2]:
        raise ValueError("dY does not match the output dimension")
    return S1, U1, U2, S2


def forward(x, S1, U1, U2, S2, b=None):
    """T1."""
    x = _f64(x)
    S1, U1, U2, S2 = _check(x.shape[1], None, S1, U1, U2, S2)
    l = S1.shape[0]
    acc = np.zeros((x.shape[0], U1.shape[2]), dtype=np.float64)
    for i in range(l):
        acc += (x @ S1[i]) @ U1[i]
        acc += (x @ U2[i]) @ S2[i].T
    y = acc / (2.0 * l)
    if b is not None:
        y = y + _f64(b)[None, :]
    return y


def grad_input(dY, S1, U1, U2, S2):
    """T2."""
    dY = _f64(dY)
    S1, U1, U2, S2 = _check(None, dY.shape[1], S1, U1, U2, S2)
    l = S1.shape[0]
    acc = np.zeros((dY.shape[0], S1.shape[1]), dtype=np.float64)
    for i in range(l):
        acc += (dY @ U1[i].T) @ S1[i].T
        acc += (dY @ S2[i]) @ U2[i].T
    return acc / (2.0 * l)


def grad_second_stage(x, S1, dY):
    """T3: dU1 [l, k, out]."""
    x, dY, S1 = _f64(x), _f64(dY), _f64(S1)
    l = S1.shape[0]
    dU1 = np.empty((l, S1.shape[2], dY.shape[1]), dtype=np.float64)
    for i in range(l):
        dU1[i] = (x @ S1[i]).T @ dY / (2.0 * l)
    return dU1


def grad_first_stage(x, S2, dY):
    """T4: dU2 [l, in, k]."""
    x, dY, S2 = _f64(x), _f64(dY), _f64(S2)
    l = S2.shape[0]
    dU2 = np.empty((l, x.shape[1], S2.shape[2]), dtype=np.float64)
    for i in range(l):
        dU2[i] = x.T @ (dY @ S2[i]) / (2.0 * l)
    return dU2


def grad_bias(dY):
    """T5."""
    return _f64(dY).sum(axis=0)


def stored_numbers(d_in, d_out, l, k):
    """Numbers the layer stores (fixed and learned, bias aside): the left-hand side of
    the paper's size rule."""
    return 2 * l * k * (d_in + d_out)


def concatenated(S1, U1, U2, S2):
    """Stage matrices of the equivalent chain with 2 l terms of rank k, in the one-sided
    oracle's conventions: S [2l, in, k] = S1 terms then U2 terms, U [2l, k, out] = U1
    terms then S2^T terms.  (Layout helper for the tests; no arithmetic.)"""
    S1, U1, U2, S2 = _check(None, None, S1, U1, U2, S2)
    S = np.concatenate([S1, U2], axis=0)
    U = np.concatenate([U1, np.transpose(S2, (0, 2, 1))], axis=0)
    return S, U
