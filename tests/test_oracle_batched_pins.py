"""Pins for the oracle's shared-input functions (matmul_batched, silu, gate_up): closed forms,
library functions other than the one the oracle calls, scalar brute force, and the algebraic
identity that several layers are ONE layer with stacked rows and block-diagonal factors.

Passages: every linear layer of a block carries its own quantised weight and factors (Sec. 4.3);
module list Q, K, V, O, Gate, Up, Down (Appendix A, Table 7); W_hat = Q (.) (BA) (Sec. 3.3).
"""
import math
import warnings

import numpy as np
import pytest

from oracle import lords_oracle as onp
from tests.helpers import pack_codes_py


def layer(rng, bits, N, K, r):
    q = rng.integers(0, 1 << bits, size=(N, K))
    return q, pack_codes_py(q, bits), rng.standard_normal((N, r)).astype(np.float32), \
        rng.standard_normal((r, K)).astype(np.float32)


# ---------------------------------------------------------------- silu
def test_silu_known_values():
    # sigma(1) = 0.731058578630004879..., so silu(1) = that, silu(-1) = -(1 - that)
    assert onp.silu(0.0) == 0.0
    assert abs(float(onp.silu(1.0)) - 0.7310585786300049) < 1e-15
    assert abs(float(onp.silu(-1.0)) + 0.2689414213699951) < 1e-15
    # ln 3: sigma = 3/4
    assert abs(float(onp.silu(math.log(3.0))) - 0.75 * math.log(3.0)) < 1e-15
    assert abs(float(onp.silu(-math.log(3.0))) + 0.25 * math.log(3.0)) < 1e-15


def test_silu_against_tanh_form_and_oddness():
    x = np.linspace(-30, 30, 2001)
    via_tanh = np.array([v * 0.5 * (1.0 + math.tanh(0.5 * v)) for v in x])
    np.testing.assert_allclose(onp.silu(x), via_tanh, rtol=1e-13, atol=1e-15)
    # sigma(x) + sigma(-x) = 1  =>  silu(x) - silu(-x) = x
    np.testing.assert_allclose(onp.silu(x) - onp.silu(-x), x, rtol=0, atol=1e-14)


def test_silu_extremes_do_not_overflow():
    with warnings.catch_warnings():
        warnings.simplefilter("error")
        big = onp.silu(np.array([800.0, -800.0, 1e300, -1e300]))
    assert big[0] == 800.0 and big[2] == 1e300
    assert big[1] == 0.0 and big[3] == 0.0
    # minimum of silu: about -0.2784645 at x about -1.2784645
    x = np.linspace(-3, 0, 300001)
    y = onp.silu(x)
    assert abs(y.min() + 0.2784645427610738) < 1e-9
    assert abs(x[y.argmin()] + 1.2784645427610738) < 2e-5


# ---------------------------------------------------------------- gate_up
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gate_up_brute_force(bits):
    rng = np.random.default_rng([11, bits])
    N, K, r, M = 5, 32, 3, 3
    C = rng.standard_normal(1 << bits).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float32)
    qg, cg, Bg, Ag = layer(rng, bits, N, K, r)
    qu, cu, Bu, Au = layer(rng, bits, N, K, r)
    got = onp.gate_up(X, (cg, Bg, Ag), (cu, Bu, Au), C, bits)
    for m in range(M):
        for n in range(N):
            g = u = 0.0
            for k in range(K):
                sg = sum(float(Bg[n, j]) * float(Ag[j, k]) for j in range(r))
                su = sum(float(Bu[n, j]) * float(Au[j, k]) for j in range(r))
                g += float(X[m, k]) * float(C[qg[n, k]]) * sg
                u += float(X[m, k]) * float(C[qu[n, k]]) * su
            want = g / (1.0 + math.exp(-g)) * u
            assert abs(got[m, n] - want) <= 1e-11 * max(1.0, abs(want)), (m, n)


def test_gate_up_identity_activations():
    # X = I: G = W_gate^T, U = W_up^T, so H[m][n] = silu(Wg[n][m]) * Wu[n][m]
    rng = np.random.default_rng(12)
    bits, N, K, r = 4, 7, 32, 2
    C = rng.standard_normal(16).astype(np.float32)
    _, cg, Bg, Ag = layer(rng, bits, N, K, r)
    _, cu, Bu, Au = layer(rng, bits, N, K, r)
    H = onp.gate_up(np.eye(K, dtype=np.float32), (cg, Bg, Ag), (cu, Bu, Au), C, bits)
    Wg, Wu = onp.dequant(cg, C, Bg, Ag, bits), onp.dequant(cu, C, Bu, Au, bits)
    want = np.vectorize(lambda g, u: g / (1.0 + math.exp(-g)) * u)(Wg, Wu).T
    np.testing.assert_allclose(H, want, rtol=1e-12, atol=1e-14)


def test_gate_up_roles_are_not_interchangeable():
    # a swapped gate and up, or an activation applied to the wrong side, changes the result
    rng = np.random.default_rng(13)
    bits, N, K, r, M = 3, 6, 64, 2, 4
    C = rng.standard_normal(8).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float32)
    _, cg, Bg, Ag = layer(rng, bits, N, K, r)
    _, cu, Bu, Au = layer(rng, bits, N, K, r)
    H = onp.gate_up(X, (cg, Bg, Ag), (cu, Bu, Au), C, bits)
    Hs = onp.gate_up(X, (cu, Bu, Au), (cg, Bg, Ag), C, bits)
    assert onp.rel_fro(Hs, H) > 0.1
    # zero up-projection (all-zero B) gives zero whatever the gate is; zero gate gives silu(0) = 0
    Z = np.zeros_like(Bu)
    assert np.all(onp.gate_up(X, (cg, Bg, Ag), (cu, Z, Au), C, bits) == 0.0)
    assert np.all(onp.gate_up(X, (cg, Z, Ag), (cu, Bu, Au), C, bits) == 0.0)


# ---------------------------------------------------------------- matmul_batched
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_batched_is_one_layer_with_stacked_rows_and_block_diagonal_factors(bits):
    # rows of all layers stacked; B block-diagonal over the layers' rank columns, A stacked:
    # (B_cat A_cat)[rows of layer l] = B_l A_l, so ONE single-layer product gives every Y_l.
    rng = np.random.default_rng([14, bits])
    K, M = 64, 3
    shapes = [(5, 2), (3, 4), (8, 1)]                 # (N_l, r_l)
    C = rng.standard_normal(1 << bits).astype(np.float32)
    X = rng.standard_normal((M, K)).astype(np.float32)
    layers = [layer(rng, bits, N, K, r) for (N, r) in shapes]
    got = onp.matmul_batched(X, [(c, B, A) for (_, c, B, A) in layers], C, bits)
    rt = sum(r for _, r in shapes)
    Bcat = np.zeros((sum(n for n, _ in shapes), rt), dtype=np.float32)
    n0 = j0 = 0
    for (N, r), (_, _, B, _) in zip(shapes, layers):
        Bcat[n0:n0 + N, j0:j0 + r] = B
        n0 += N
        j0 += r
    Acat = np.concatenate([A for (_, _, _, A) in layers], axis=0)
    ccat = np.concatenate([c for (_, c, _, _) in layers], axis=0)
    Ycat = onp.matmul(X, ccat, C, Bcat, Acat, bits)
    n0 = 0
    for (N, _), Y in zip(shapes, got):
        assert Y.shape == (M, N)
        np.testing.assert_allclose(Y, Ycat[:, n0:n0 + N], rtol=1e-12, atol=1e-12)
        n0 += N


def test_batched_order_and_count():
    rng = np.random.default_rng(15)
    bits, K = 4, 32
    C = rng.standard_normal(16).astype(np.float32)
    X = rng.standard_normal((2, K)).astype(np.float32)
    a, b = layer(rng, bits, 4, K, 2), layer(rng, bits, 6, K, 2)
    Y = onp.matmul_batched(X, [(a[1], a[2], a[3]), (b[1], b[2], b[3])], C, bits)
    assert [y.shape for y in Y] == [(2, 4), (2, 6)]
    Yr = onp.matmul_batched(X, [(b[1], b[2], b[3]), (a[1], a[2], a[3])], C, bits)
    np.testing.assert_array_equal(Y[0], Yr[1])
    np.testing.assert_array_equal(Y[1], Yr[0])
    assert onp.matmul_batched(X, [], C, bits) == []
