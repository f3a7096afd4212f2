"""Pins of the two-sided oracle (oracle/sklinear_two_sided.py): everything here is
fixed by the mathematics or by the paper's size rule, none of it by the oracle."""
import os

import numpy as np
import pytest

from oracle import sklinear as O1
from oracle import sklinear_two_sided as O2

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "size_rule.txt")


def rand_case(seed, T, d_in, d_out, l, k):
    r = np.random.default_rng(seed)
    return dict(
        x=r.standard_normal((T, d_in)),
        S1=r.standard_normal((l, d_in, k)) / np.sqrt(k),
        U1=r.standard_normal((l, k, d_out)),
        U2=r.standard_normal((l, d_in, k)),
        S2=r.standard_normal((l, d_out, k)) / np.sqrt(k),
        b=r.standard_normal(d_out),
        dY=r.standard_normal((T, d_out)),
    )


def loss_loops(c, x=None, U1=None, U2=None, b=None):
    """L = sum(dY * y) from the definition, scalar loops only (tiny shapes)."""
    x = c["x"] if x is None else x
    U1 = c["U1"] if U1 is None else U1
    U2 = c["U2"] if U2 is None else U2
    b = c["b"] if b is None else b
    S1, S2, dY = c["S1"], c["S2"], c["dY"]
    l, d_in, k = S1.shape
    d_out = U1.shape[2]
    total = 0.0
    for t in range(x.shape[0]):
        for o in range(d_out):
            acc = 0.0
            for i in range(l):
                for j in range(k):
                    z1 = sum(x[t, a] * S1[i, a, j] for a in range(d_in))
                    z2 = sum(x[t, a] * U2[i, a, j] for a in range(d_in))
                    acc += z1 * U1[i, j, o] + z2 * S2[i, o, j]
            total += dY[t, o] * (acc / (2 * l) + b[o])
    return total


def test_identity_sketches_give_the_mean_of_two_dense_layers():
    r = np.random.default_rng(0)
    n, T = 7, 5
    x, U1, U2, b = r.standard_normal((T, n)), r.standard_normal((1, n, n)), r.standard_normal((1, n, n)), r.standard_normal(n)
    I = np.eye(n)[None]
    y = O2.forward(x, I, U1, U2, I, b)
    assert np.allclose(y, x @ (U1[0] + U2[0]) / 2 + b, rtol=0, atol=1e-13)
    dY = r.standard_normal((T, n))
    assert np.allclose(O2.grad_input(dY, I, U1, U2, I), dY @ (U1[0] + U2[0]).T / 2, atol=1e-13)
    assert np.allclose(O2.grad_second_stage(x, I, dY)[0], x.T @ dY / 2, atol=1e-13)
    assert np.allclose(O2.grad_first_stage(x, I, dY)[0], x.T @ dY / 2, atol=1e-13)


@pytest.mark.parametrize("shape", [(3, 4, 5, 1, 2), (2, 5, 3, 3, 2)])
def test_gradients_by_central_differences(shape):
    """L is linear in x, U1, U2 and b separately, so central differences of a loop-only
    loss are exact up to rounding: every entry of every gradient."""
    c = rand_case(1, *shape)
    h = 0.5
    args = (c["S1"], c["U1"], c["U2"], c["S2"])
    got = dict(x=O2.grad_input(c["dY"], *args), U1=O2.grad_second_stage(c["x"], c["S1"], c["dY"]),
               U2=O2.grad_first_stage(c["x"], c["S2"], c["dY"]), b=O2.grad_bias(c["dY"]))
    for name in ("x", "U1", "U2", "b"):
        base = c[name]
        for idx in np.ndindex(base.shape):
            up, dn = base.copy(), base.copy()
            up[idx] += h
            dn[idx] -= h
            fd = (loss_loops(c, **{name: up}) - loss_loops(c, **{name: dn})) / (2 * h)
            assert abs(fd - got[name][idx]) <= 1e-9 * max(1.0, abs(fd)), (name, idx)


@pytest.mark.parametrize("shape", [(6, 5, 4, 1, 3), (9, 8, 11, 3, 2)])
def test_equals_one_sided_layer_on_concatenated_stage_matrices(shape):
    """[S1 | U2] then [U1 ; S2^T] with 2 l terms: the one-sided oracle (pinned on its own)
    must give the same y and dX, its factor gradient holds dU1 in the first l terms, and the
    first-stage gradient is x^T (dY B^T) restricted to the U2 columns."""
    c = rand_case(2, *shape)
    l = shape[3]
    S, U = O2.concatenated(c["S1"], c["U1"], c["U2"], c["S2"])
    args = (c["S1"], c["U1"], c["U2"], c["S2"])
    assert np.allclose(O2.forward(c["x"], *args, c["b"]), O1.forward(c["x"], S, U, c["b"]), atol=1e-12)
    assert np.allclose(O2.grad_input(c["dY"], *args), O1.grad_input(c["dY"], S, U), atol=1e-12)
    dU = O1.grad_factors(c["x"], S, c["dY"])
    assert np.allclose(O2.grad_second_stage(c["x"], c["S1"], c["dY"]), dU[:l], atol=1e-12)
    G = np.stack([c["dY"] @ U[l + i].T for i in range(l)])          # [l, T, k]
    want = np.stack([c["x"].T @ G[i] for i in range(l)]) / (2 * l)
    assert np.allclose(O2.grad_first_stage(c["x"], c["S2"], c["dY"]), want, atol=1e-12)


def test_adjoint_identity():
    c = rand_case(3, 40, 24, 36, 2, 8)
    args = (c["S1"], c["U1"], c["U2"], c["S2"])
    y = O2.forward(c["x"], *args, c["b"])
    lhs = np.sum(c["dY"] * (y - c["b"]))
    assert np.isclose(lhs, np.sum(O2.grad_input(c["dY"], *args) * c["x"]), rtol=1e-12)
    rhs = np.sum(O2.grad_second_stage(c["x"], c["S1"], c["dY"]) * c["U1"]) + \
        np.sum(O2.grad_first_stage(c["x"], c["S2"], c["dY"]) * c["U2"])
    assert np.isclose(lhs, rhs, rtol=1e-12)


def test_stored_numbers_are_the_left_side_of_the_papers_size_rule():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert rows
    for d_in, d_out, l, k, lhs, rhs, skipped in (map(int, r) for r in rows):
        assert O2.stored_numbers(d_in, d_out, l, k) == lhs
    c = rand_case(0, 1, 16, 32, 2, 4)
    assert sum(c[n].size for n in ("S1", "U1", "U2", "S2")) == O2.stored_numbers(16, 32, 2, 4)


def test_expected_value_over_gaussian_sketches():
    """U1_i = S1_i^T W^T and U2_i = W^T S2_i make every term unbiased for x W^T when the
    sketch entries are N(0, 1/k): the mean over many draws approaches the dense layer."""
    r = np.random.default_rng(5)
    d_in, d_out, l, k, T = 6, 5, 2, 3, 4
    W = r.standard_normal((d_out, d_in))
    x = r.standard_normal((T, d_in))
    n = 4000
    ys = np.empty((n, T, d_out))
    for s in range(n):
        S1 = r.standard_normal((l, d_in, k)) / np.sqrt(k)
        S2 = r.standard_normal((l, d_out, k)) / np.sqrt(k)
        U1 = np.stack([S1[i].T @ W.T for i in range(l)])
        U2 = np.stack([W.T @ S2[i] for i in range(l)])
        ys[s] = O2.forward(x, S1, U1, U2, S2)
    mean, sem = ys.mean(axis=0), ys.std(axis=0, ddof=1) / np.sqrt(n)
    assert np.all(np.abs(mean - x @ W.T) <= 4.5 * sem)
