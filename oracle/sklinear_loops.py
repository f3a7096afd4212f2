"""Brute-force SKLinear in pure Python loops, for tiny inputs only.

TEST INFRASTRUCTURE ONLY.  Evaluates the layer of paper Sec. 3.1 entry by
entry -- no matrix library, no vectorisation -- so that the numpy oracle in
``oracle/sklinear.py`` can be pinned against something that cannot share an
indexing or transposition mistake with it.  Python floats are IEEE fp64.

Conventions as in ``oracle/sklinear.py``: x [T][in], S [l][in][k],
U [l][k][out], b [out] or None.
"""
from __future__ import annotations


def forward(x, S, U, b=None):
    T, d_in = len(x), len(x[0])
    l, k, d_out = len(S), len(S[0][0]), len(U[0][0])
    y = [[0.0] * d_out for _ in range(T)]
    for t in range(T):
        for o in range(d_out):
            total = 0.0
            for i in range(l):
                for j in range(k):
                    z = 0.0                      # (x . S_i)[t, j]
                    for a in range(d_in):
                        z += x[t][a] * S[i][a][j]
                    total += z * U[i][j][o]
            y[t][o] = total / l + (b[o] if b is not None else 0.0)
    return y


def loss(x, S, U, b, dY):
    """L = sum over (t, o) of dY[t][o] * y[t][o]."""
    y = forward(x, S, U, b)
    return sum(dY[t][o] * y[t][o] for t in range(len(y)) for o in range(len(y[0])))


def grad_input(dY, S, U):
    T, d_out = len(dY), len(dY[0])
    l, d_in, k = len(S), len(S[0]), len(S[0][0])
    dX = [[0.0] * d_in for _ in range(T)]
    for t in range(T):
        for a in range(d_in):
            total = 0.0
            for i in range(l):
                for j in range(k):
                    g = 0.0                      # (dY . U_i^T)[t, j]
                    for o in range(d_out):
                        g += dY[t][o] * U[i][j][o]
                    total += g * S[i][a][j]
            dX[t][a] = total / l
    return dX


def grad_factors(x, S, dY):
    T, d_in, d_out = len(x), len(x[0]), len(dY[0])
    l, k = len(S), len(S[0][0])
    dU = [[[0.0] * d_out for _ in range(k)] for _ in range(l)]
    for i in range(l):
        for j in range(k):
            for o in range(d_out):
                total = 0.0
                for t in range(T):
                    z = 0.0
                    for a in range(d_in):
                        z += x[t][a] * S[i][a][j]
                    total += z * dY[t][o]
                dU[i][j][o] = total / l
    return dU


def grad_bias(dY):
    return [sum(dY[t][o] for t in range(len(dY))) for o in range(len(dY[0]))]
