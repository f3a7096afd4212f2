"""Plain fp64 oracle of the sketched linear layer (SKLinear).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

What the layer computes (paper Sec. 3.1, "During Development use-case"): the
output is the *average* over ``num_terms`` (= l) sketched matrix products,
each of rank ``low_rank`` (= k), and the layer is a drop-in for a dense linear
layer, hence a bias that is added once.  Written out, with fixed random
sketches S_i (in x k) and learned factors U_i (k x out):

    y = (1/l) * sum_i (x . S_i) . U_i + b                               (D1)

The paper prints no gradient; D2-D4 below are the exact derivatives of the
scalar  L = sum(dY * y)  with respect to x, U_i and b.  S_i is fixed, so it has
no gradient.

    dX   = (1/l) * sum_i (dY . U_i^T) . S_i^T                            (D2)
    dU_i = (1/l) * (x . S_i)^T . dY                                      (D3)
    db   = sum over tokens of dY                                         (D4)

Every function takes the terms one at a time, in the order of the definition,
with one library matmul per product and fp64 throughout.  The l sketches are
never concatenated here: that the concatenated form gives the same numbers is
something the tests check, not something the oracle assumes.

Array conventions: x [T, in], S [l, in, k], U [l, k, out], b [out] or None,
y and dY [T, out], dX [T, in], dU [l, k, out], db [out].

Pinned (tests/test_oracle_pins.py) by: the dense special case S = I, the
concatenated-GEMM identity, central finite differences of a loop-only forward,
adjoint (Euler) identities, scaling/permutation invariants, the expectation
and variance of the Gaussian sketch estimator, and a pure-Python brute force.
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _check(x_cols, S, U=None):
    S = _f64(S)
    if S.ndim != 3:
        raise ValueError("S must be [l, in, k]")
    if x_cols is not None and S.shape[1] != x_cols:
        raise ValueError("feature dimension of x does not match S")
    if U is not None:
        U = _f64(U)
        if U.ndim != 3 or U.shape[0] != S.shape[0] or U.shape[1] != S.shape[2]:
            raise ValueError("U must be [l, k, out] with the same l and k as S")
    return S, U


def forward(x, S, U, b=None):
    """D1 (Sec. 3.1): average of l rank-k sketched products, plus bias."""
    x = _f64(x)
    S, U = _check(x.shape[1], S, U)
    l = S.shape[0]
    acc = np.zeros((x.shape[0], U.shape[2]), dtype=np.float64)
    for i in range(l):
        z_i = x @ S[i]            # sketch the input: [T, k]
        acc += z_i @ U[i]         # expand with the learned factor: [T, out]
    y = acc / l
    if b is not None:
        y = y + _f64(b)[None, :]
    return y


def grad_input(dY, S, U):
    """D2: derivative of sum(dY * y) with respect to x."""
    dY = _f64(dY)
    S, U = _check(None, S, U)
    if dY.shape[1] != U.shape[2]:
        raise ValueError("dY columns must equal out")
    l = S.shape[0]
    acc = np.zeros((dY.shape[0], S.shape[1]), dtype=np.float64)
    for i in range(l):
        g_i = dY @ U[i].T         # [T, k]
        acc += g_i @ S[i].T       # [T, in]
    return acc / l


def grad_factors(x, S, dY):
    """D3: derivative of sum(dY * y) with respect to each U_i; [l, k, out]."""
    x = _f64(x)
    dY = _f64(dY)
    S, _ = _check(x.shape[1], S)
    if dY.shape[0] != x.shape[0]:
        raise ValueError("x and dY must have the same number of tokens")
    l = S.shape[0]
    dU = np.empty((l, S.shape[2], dY.shape[1]), dtype=np.float64)
    for i in range(l):
        z_i = x @ S[i]            # recomputed, as the layer does not keep it
        dU[i] = (z_i.T @ dY) / l
    return dU


def grad_bias(dY):
    """D4: derivative of sum(dY * y) with respect to b."""
    return _f64(dY).sum(axis=0)


# ---------------------------------------------------------------------------
# Size accounting (Sec. 4.1, the rule that decides which benchmark points the
# paper skips).
# ---------------------------------------------------------------------------

def stored_numbers(d_in, d_out, l, k):
    """Numbers held by the one-sided layer: l sketches in x k, l factors k x out."""
    return l * k * (d_in + d_out)


def learned_numbers(d_in, d_out, l, k, bias=True):
    """Trainable numbers: the factors U_i and the bias (the sketches are fixed)."""
    return l * k * d_out + (d_out if bias else 0)


def paper_skips(d_in, d_out, l, k):
    """True when Sec. 4.1's inequality 2 l k (d_in + d_out) > d_in d_out holds."""
    return 2 * l * k * (d_in + d_out) > d_in * d_out
