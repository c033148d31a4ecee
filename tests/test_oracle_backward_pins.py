"""Pins for the oracle's backward functions (gradients with respect to X and to the scale factors
B and A, Sec. 3.4): central differences of the oracle's own FORWARD function (which is pinned
elsewhere), the adjoint identity, scalar brute force, and the block-wise special case (Sec. 3.1)
where dB is a per-block sum.
"""
import numpy as np
import pytest

from oracle import lords_oracle as onp
from tests.helpers import pack_codes_py


def case(bits, N=6, K=32, r=3, M=4, seed=0):
    rng = np.random.default_rng([41, seed, bits])
    q = rng.integers(0, 1 << bits, size=(N, K))
    return dict(q=q, codes=pack_codes_py(q, bits), C=rng.standard_normal(1 << bits),
                B=rng.standard_normal((N, r)), A=rng.standard_normal((r, K)),
                X=rng.standard_normal((M, K)), dY=rng.standard_normal((M, N)), bits=bits)


def loss(c, X=None, B=None, A=None):
    """<dY, Y>: a scalar whose gradient with respect to Y is dY."""
    Y = onp.matmul(c["X"] if X is None else X, c["codes"], c["C"], c["B"] if B is None else B,
                   c["A"] if A is None else A, c["bits"])
    return float(np.sum(c["dY"] * Y))


def central_difference(f, x0, h=1e-6):
    g = np.zeros_like(x0)
    for idx in np.ndindex(*x0.shape):
        xp, xm = x0.copy(), x0.copy()
        xp[idx] += h
        xm[idx] -= h
        g[idx] = (f(xp) - f(xm)) / (2 * h)
    return g


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gradients_match_central_differences_of_the_forward(bits):
    # the loss is linear in X and bilinear in (B, A): central differences are exact up to rounding
    c = case(bits)
    dX = onp.backward_input(c["dY"], c["codes"], c["C"], c["B"], c["A"], bits)
    dB, dA = onp.backward_factors(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], bits)
    np.testing.assert_allclose(dX, central_difference(lambda v: loss(c, X=v), c["X"]), rtol=1e-7, atol=1e-7)
    np.testing.assert_allclose(dB, central_difference(lambda v: loss(c, B=v), c["B"]), rtol=1e-7, atol=1e-7)
    np.testing.assert_allclose(dA, central_difference(lambda v: loss(c, A=v), c["A"]), rtol=1e-7, atol=1e-7)


def test_adjoint_identity():
    # <dY, X W^T> = <dY W, X>
    c = case(4, N=9, K=64, r=4, M=5, seed=1)
    Y = onp.matmul(c["X"], c["codes"], c["C"], c["B"], c["A"], 4)
    dX = onp.backward_input(c["dY"], c["codes"], c["C"], c["B"], c["A"], 4)
    assert abs(np.sum(c["dY"] * Y) - np.sum(dX * c["X"])) <= 1e-10 * abs(np.sum(c["dY"] * Y))


def test_scalar_brute_force():
    c = case(3, N=4, K=32, r=2, M=3, seed=2)
    N, K, r, M = 4, 32, 2, 3
    dX = onp.backward_input(c["dY"], c["codes"], c["C"], c["B"], c["A"], 3)
    dB, dA = onp.backward_factors(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], 3)
    lvl = lambda n, k: c["C"][c["q"][n, k]]
    for m in range(M):
        for k in range(K):
            want = sum(c["dY"][m, n] * lvl(n, k) * sum(c["B"][n, j] * c["A"][j, k] for j in range(r)) for n in range(N))
            assert abs(dX[m, k] - want) < 1e-11
    for n in range(N):
        for j in range(r):
            want = sum(lvl(n, k) * c["A"][j, k] * sum(c["dY"][m, n] * c["X"][m, k] for m in range(M)) for k in range(K))
            assert abs(dB[n, j] - want) < 1e-10
    for j in range(r):
        for k in range(K):
            want = sum(c["B"][n, j] * lvl(n, k) * sum(c["dY"][m, n] * c["X"][m, k] for m in range(M)) for n in range(N))
            assert abs(dA[j, k] - want) < 1e-10


def test_blockwise_special_case():
    # A = block indicator (Sec. 3.1 in matrix form): the gradient of a block's scale is the sum over the
    # block of level * dLoss/dW_hat, and dA[j][k] only sees the scales of block j
    c = case(4, N=5, K=64, r=4, M=3, seed=3)
    g = 16
    A = np.zeros((4, 64))
    for j in range(4):
        A[j, j * g:(j + 1) * g] = 1.0
    dB, dA = onp.backward_factors(c["dY"], c["X"], c["codes"], c["C"], c["B"], A, 4)
    Gw = c["dY"].T @ c["X"]
    P = c["C"][c["q"]] * Gw
    np.testing.assert_allclose(dB, P.reshape(5, 4, g).sum(axis=2), rtol=1e-12, atol=1e-12)
    for j in range(4):
        np.testing.assert_allclose(dA[j], c["B"][:, j] @ P, rtol=1e-12, atol=1e-12)


def test_planted_mistakes_are_caught():
    # a transposed operand or a dropped level factor must fail the central-difference pin
    c = case(4, seed=4)
    dB, dA = onp.backward_factors(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], 4)
    fd_B = central_difference(lambda v: loss(c, B=v), c["B"])
    G = c["dY"].T @ c["X"]
    wrong_no_level = G @ c["A"].T
    wrong_role = (c["C"][c["q"]] * G) @ c["A"].T * 0 + c["B"]           # anything else of the same shape
    assert not np.allclose(wrong_no_level, fd_B, rtol=1e-3, atol=1e-3)
    assert not np.allclose(wrong_role, fd_B, rtol=1e-3, atol=1e-3)
    assert np.allclose(dB, fd_B, rtol=1e-7, atol=1e-7)


def test_restricted_forms_match_the_full_ones():
    c = case(3, N=12, K=64, r=3, M=5, seed=5)
    dX = onp.backward_input(c["dY"], c["codes"], c["C"], c["B"], c["A"], 3)
    dB, dA = onp.backward_factors(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], 3)
    cols, rows = [0, 7, 63, 31], [11, 0, 5]
    np.testing.assert_allclose(onp.backward_input_cols(c["dY"], c["codes"], c["C"], c["B"], c["A"], 3, cols), dX[:, cols],
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(onp.backward_factors_rows(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], 3, rows),
                               dB[rows], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(onp.backward_factors_cols(c["dY"], c["X"], c["codes"], c["C"], c["B"], c["A"], 3, cols),
                               dA[:, cols], rtol=1e-12, atol=1e-12)
