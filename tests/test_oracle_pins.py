"""Pins of the fp64 oracle against things other than itself (CPU only).

The paper prints no worked numerical example of the layer, so the oracle is
pinned by closed forms, brute force, finite differences, invariants and the
statistics that Sec. 3.1 alludes to ("closer to the expected value").
"""
import os

import numpy as np
import pytest

from oracle import sklinear as O
from oracle import sklinear_loops as L

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_case(seed, T, d_in, d_out, l, k):
    r = np.random.default_rng(seed)
    return dict(
        x=r.standard_normal((T, d_in)),
        S=r.standard_normal((l, d_in, k)) / np.sqrt(k),
        U=r.standard_normal((l, k, d_out)),
        b=r.standard_normal(d_out),
        dY=r.standard_normal((T, d_out)),
    )


SHAPES = [(3, 4, 5, 2, 3), (1, 2, 2, 1, 1), (4, 6, 3, 3, 5), (5, 3, 7, 1, 4)]


# --- P0: brute force ---------------------------------------------------------
@pytest.mark.parametrize("shape", SHAPES)
def test_matches_pure_python_brute_force(shape):
    c = rand_case(11, *shape)
    tl = {n: a.tolist() for n, a in c.items()}
    np.testing.assert_allclose(O.forward(c["x"], c["S"], c["U"], c["b"]),
                               np.array(L.forward(tl["x"], tl["S"], tl["U"], tl["b"])),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.forward(c["x"], c["S"], c["U"], None),
                               np.array(L.forward(tl["x"], tl["S"], tl["U"], None)),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.grad_input(c["dY"], c["S"], c["U"]),
                               np.array(L.grad_input(tl["dY"], tl["S"], tl["U"])),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.grad_factors(c["x"], c["S"], c["dY"]),
                               np.array(L.grad_factors(tl["x"], tl["S"], tl["dY"])),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.grad_bias(c["dY"]), np.array(L.grad_bias(tl["dY"])),
                               rtol=0, atol=1e-12)


# --- P1: l = 1, S = I is the textbook dense layer ----------------------------
def test_identity_sketch_is_dense_linear_layer():
    T, d, d_out = 7, 6, 9
    c = rand_case(3, T, d, d_out, 1, d)
    S = np.eye(d)[None]
    W = c["U"][0]                                   # y = x W + b
    np.testing.assert_allclose(O.forward(c["x"], S, c["U"], c["b"]),
                               c["x"] @ W + c["b"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(O.grad_input(c["dY"], S, c["U"]),
                               c["dY"] @ W.T, rtol=0, atol=1e-13)
    np.testing.assert_allclose(O.grad_factors(c["x"], S, c["dY"])[0],
                               c["x"].T @ c["dY"], rtol=0, atol=1e-13)
    # hand-worked 1x2 example: x=[1,2], U=[[3,4],[5,6]], b=[.5,-.5] -> [13.5, 15.5]
    y = O.forward([[1.0, 2.0]], np.eye(2)[None], [[[3.0, 4.0], [5.0, 6.0]]], [0.5, -0.5])
    np.testing.assert_array_equal(y, [[13.5, 15.5]])


def test_hand_worked_two_term_example():
    # in=1, k=1, out=1: y = (x*s1*u1 + x*s2*u2)/2 + b
    x = [[2.0]]
    S = [[[3.0]], [[5.0]]]
    U = [[[7.0]], [[-1.0]]]
    y = O.forward(x, S, U, [0.25])
    assert y[0, 0] == (2 * 3 * 7 + 2 * 5 * -1) / 2 + 0.25          # 16.25
    dY = [[4.0]]
    assert O.grad_input(dY, S, U)[0, 0] == 4 * (7 * 3 + -1 * 5) / 2  # 32
    dU = O.grad_factors(x, S, dY)
    assert dU[0, 0, 0] == 2 * 3 * 4 / 2 and dU[1, 0, 0] == 2 * 5 * 4 / 2
    assert O.grad_bias([[4.0], [1.5]])[0] == 5.5


# --- P2: the sum of l terms is one concatenated contraction ------------------
@pytest.mark.parametrize("shape", SHAPES + [(9, 12, 10, 3, 5)])
def test_concatenation_identity(shape):
    T, d_in, d_out, l, k = shape
    c = rand_case(5, *shape)
    S_cat = np.transpose(c["S"], (1, 0, 2)).reshape(d_in, l * k)
    U_cat = c["U"].reshape(l * k, d_out)
    np.testing.assert_allclose(O.forward(c["x"], c["S"], c["U"], c["b"]),
                               (c["x"] @ S_cat) @ U_cat / l + c["b"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.grad_input(c["dY"], c["S"], c["U"]),
                               (c["dY"] @ U_cat.T) @ S_cat.T / l, rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.grad_factors(c["x"], c["S"], c["dY"]).reshape(l * k, d_out),
                               (c["x"] @ S_cat).T @ c["dY"] / l, rtol=0, atol=1e-12)


# --- P3: finite differences of the loop-only loss ----------------------------
@pytest.mark.parametrize("shape", [(3, 4, 5, 2, 3), (2, 3, 2, 3, 2)])
def test_gradients_by_central_differences(shape):
    c = rand_case(7, *shape)
    x, S, U, b, dY = (c[n] for n in ("x", "S", "U", "b", "dY"))

    def loss(x_, U_, b_):
        return L.loss(x_.tolist(), S.tolist(), U_.tolist(), b_.tolist(), dY.tolist())

    h = 0.5  # L is linear in each of x, U, b separately: any step is exact
    dX = O.grad_input(dY, S, U)
    for idx in np.ndindex(*x.shape):
        e = np.zeros_like(x); e[idx] = h
        fd = (loss(x + e, U, b) - loss(x - e, U, b)) / (2 * h)
        assert abs(fd - dX[idx]) < 1e-9
    dU = O.grad_factors(x, S, dY)
    for idx in np.ndindex(*U.shape):
        e = np.zeros_like(U); e[idx] = h
        fd = (loss(x, U + e, b) - loss(x, U - e, b)) / (2 * h)
        assert abs(fd - dU[idx]) < 1e-9
    db = O.grad_bias(dY)
    for o in range(b.shape[0]):
        e = np.zeros_like(b); e[o] = h
        fd = (loss(x, U, b + e) - loss(x, U, b - e)) / (2 * h)
        assert abs(fd - db[o]) < 1e-9


# --- P4: adjoint (Euler) identities ------------------------------------------
def test_adjoint_identities():
    c = rand_case(13, 33, 20, 17, 3, 6)
    x, S, U, b, dY = (c[n] for n in ("x", "S", "U", "b", "dY"))
    y = O.forward(x, S, U, b)
    lhs = np.sum(dY * (y - b))
    assert np.isclose(lhs, np.sum(O.grad_input(dY, S, U) * x), rtol=1e-11)
    assert np.isclose(lhs, np.sum(O.grad_factors(x, S, dY) * U), rtol=1e-11)
    assert np.isclose(np.sum(O.grad_bias(dY) * b), np.sum(dY * b[None, :]), rtol=1e-11)


# --- P5: invariants that separate an average from a sum ----------------------
def test_invariants():
    c = rand_case(17, 6, 8, 5, 3, 4)
    x, S, U, b, dY = (c[n] for n in ("x", "S", "U", "b", "dY"))
    y = O.forward(x, S, U, b)
    perm = [2, 0, 1]
    np.testing.assert_allclose(O.forward(x, S[perm], U[perm], b), y, atol=1e-12)
    # l identical copies of one term give that term's l = 1 result
    S1, U1 = S[:1], U[:1]
    np.testing.assert_allclose(O.forward(x, np.repeat(S1, 4, 0), np.repeat(U1, 4, 0), b),
                               O.forward(x, S1, U1, b), atol=1e-12)
    np.testing.assert_allclose(O.grad_input(dY, np.repeat(S1, 4, 0), np.repeat(U1, 4, 0)),
                               O.grad_input(dY, S1, U1), atol=1e-12)
    np.testing.assert_allclose(O.grad_factors(x, np.repeat(S1, 4, 0), dY).sum(0),
                               O.grad_factors(x, S1, dY)[0], atol=1e-12)
    a = 3.0
    np.testing.assert_allclose(O.forward(x, S, a * U, b) - b, a * (y - b), atol=1e-11)
    np.testing.assert_allclose(O.grad_input(dY, S, a * U), a * O.grad_input(dY, S, U), atol=1e-11)
    np.testing.assert_allclose(O.forward(a * x, S, U, b) - b, a * (y - b), atol=1e-11)
    np.testing.assert_allclose(O.grad_factors(a * x, S, dY), a * O.grad_factors(x, S, dY), atol=1e-11)
    # the bias is added once, outside the average
    np.testing.assert_allclose(O.forward(x, S, U, b) - O.forward(x, S, U, None),
                               np.broadcast_to(b, y.shape), atol=1e-12)


# --- P6: expectation and variance of the Gaussian sketch estimator -----------
@pytest.mark.parametrize("l", [1, 2, 4])
def test_expected_value_and_variance(l):
    d, k, n_seeds = 8, 4, 20000
    r = np.random.default_rng(100 + l)
    x = r.standard_normal((1, d))
    W = np.eye(d)                       # dense layer being approximated: y = x W^T + b
    b = r.standard_normal(d)
    ys = np.empty((n_seeds, d))
    for s in range(n_seeds):
        S = r.standard_normal((l, d, k)) / np.sqrt(k)          # entries N(0, 1/k)
        U = np.stack([S[i].T @ W.T for i in range(l)])          # U_i = S_i^T W^T
        ys[s] = O.forward(x, S, U, b)[0]
    want_mean = (x @ W.T + b)[0]
    want_var = (np.sum(x ** 2) + x[0] ** 2) / (l * k)           # Wishart second moment
    se = np.sqrt(want_var / n_seeds)
    assert np.all(np.abs(ys.mean(0) - want_mean) < 4.5 * se)
    assert np.all(np.abs(ys.var(0) / want_var - 1.0) < 0.10)


# --- P7: the paper's size rule ------------------------------------------------
def test_size_rule_golden():
    rows = 0
    with open(os.path.join(HERE, "golden", "size_rule.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            d_in, d_out, l, k, lhs, rhs, skipped = map(int, line.split())
            assert 2 * O.stored_numbers(d_in, d_out, l, k) == lhs
            assert d_in * d_out == rhs
            assert O.paper_skips(d_in, d_out, l, k) == bool(skipped)
            rows += 1
    assert rows >= 10
    assert O.learned_numbers(768, 3072, 2, 64) == 2 * 64 * 3072 + 3072
    assert O.learned_numbers(768, 3072, 2, 64, bias=False) == 2 * 64 * 3072


def test_shape_errors():
    c = rand_case(1, 3, 4, 5, 2, 3)
    with pytest.raises(ValueError):
        O.forward(c["x"][:, :3], c["S"], c["U"])
    with pytest.raises(ValueError):
        O.forward(c["x"], c["S"], c["U"][:1])
    with pytest.raises(ValueError):
        O.grad_factors(c["x"], c["S"], c["dY"][:2])
