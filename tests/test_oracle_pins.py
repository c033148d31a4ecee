"""Pins for the CPU oracles (numpy fp64 and plain C fp64): each check ties the
oracle to something other than itself -- hand-derived bytes, scalar brute
force, closed forms and special cases fixed by the paper or by algebra.

Paper passages: block-wise dequantisation W_b = Q_b * s_b and its matrix form
S = s (x) 1 (Sec. 3.1, Eq. 1-2); S = BA (Sec. 3.2, Eq. 3); W_hat = Q (.) (BA)
(Sec. 3.3); equivalent rank r = floor(nm / (B(n+m))) and Table 7 (Appendix A).
"""
import math
import os
import types

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import lords_inputs as li
from oracle import lords_oracle as onp
from oracle import lords_oracle_c as oc
from tests.helpers import pack_codes_py, read_packed_golden, read_rank_table

IMPLS = {"numpy": onp, "c": oc}


@pytest.fixture(params=list(IMPLS))
def impl(request):
    return IMPLS[request.param]


def small_case(bits, N=6, K=32, r=3, M=2, seed=1, signed=True):
    rng = np.random.default_rng([seed, bits, N, K, r])
    q = rng.integers(0, 1 << bits, size=(N, K))
    codes = pack_codes_py(q, bits)
    C = rng.standard_normal(1 << bits).astype(np.float32)
    B = rng.standard_normal((N, r)).astype(np.float32)
    A = rng.standard_normal((r, K)).astype(np.float32)
    if not signed:
        B, A = np.abs(B) + 0.5, np.abs(A) + 0.5
    X = rng.standard_normal((M, K)).astype(np.float32)
    return q, codes, C, B, A, X


# ---------------------------------------------------------------- unpacking
def test_unpack_hand_bytes(impl, golden_dir):
    for bits, byts, codes in read_packed_golden(os.path.join(golden_dir, "packed_bytes.txt")):
        got = impl.unpack_codes(byts[None, :], codes.size, bits)
        assert got.dtype == np.uint8
        np.testing.assert_array_equal(got[0], codes, err_msg=f"bits={bits} bytes={byts}")


@settings(max_examples=60, deadline=None)
@given(bits=st.sampled_from([2, 3, 4]), n=st.integers(1, 3), groups=st.integers(1, 3), data=st.data())
def test_unpack_inverts_independent_packer(bits, n, groups, data):
    K = 32 * groups
    q = np.array(data.draw(st.lists(st.lists(st.integers(0, (1 << bits) - 1), min_size=K, max_size=K),
                                    min_size=n, max_size=n)), dtype=np.uint8)
    codes = pack_codes_py(q, bits)
    for impl in IMPLS.values():
        np.testing.assert_array_equal(impl.unpack_codes(codes, K, bits), q)


def test_unpack_random_bytes_against_bigint(impl):
    rng = np.random.default_rng(7)
    for bits in (2, 3, 4):
        K = 96
        codes = rng.integers(0, 256, size=(5, K * bits // 8), dtype=np.uint8)
        got = impl.unpack_codes(codes, K, bits)
        for n in range(codes.shape[0]):
            big = int.from_bytes(codes[n].tobytes(), "little")
            want = [(big >> (bits * k)) & ((1 << bits) - 1) for k in range(K)]
            assert got[n].tolist() == want


# ------------------------------------------------------------ scale, dequant
def test_scale_matrix_brute_force():
    _, _, _, B, A, _ = small_case(4, N=5, K=32, r=4)
    S = onp.scale_matrix(B, A)
    for n in range(B.shape[0]):
        for k in range(A.shape[1]):
            want = math.fsum(float(B[n, j]) * float(A[j, k]) for j in range(B.shape[1]))
            assert S[n, k] == pytest.approx(want, rel=1e-14, abs=1e-300)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_dequant_brute_force(impl, bits):
    q, codes, C, B, A, _ = small_case(bits, N=4, K=32, r=3)
    W = impl.dequant(codes, C, B, A, bits)
    assert W.dtype == np.float64 and W.shape == q.shape
    for n in range(q.shape[0]):
        for k in range(q.shape[1]):
            s = math.fsum(float(B[n, j]) * float(A[j, k]) for j in range(B.shape[1]))
            assert W[n, k] == pytest.approx(float(C[q[n, k]]) * s, rel=1e-13, abs=1e-300)


@pytest.mark.parametrize("bits,group", [(4, 32), (2, 64), (3, 32), (4, 128)])
def test_blockwise_special_case_is_exact(impl, bits, group):
    """With A the 0/1 group indicator and B the block scales, LoRDS dequantisation
    IS block-wise dequantisation (Sec. 3.1: S = s (x) 1; Eq. 2: W_b = Q_b * s_b).
    One non-zero term per sum, so equality is exact in fp64."""
    cs = li.make_blockwise_case(24, 256, bits, group, seed=3, factor_dtype="f32")
    W = impl.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    big = [int.from_bytes(cs.codes[n].tobytes(), "little") for n in range(cs.N)]
    s = cs.extra["block_scales"]
    for n in range(cs.N):
        for b in range(cs.K // group):          # block b of row n shares one scale
            for t in range(group):
                k = b * group + t
                qv = (big[n] >> (bits * k)) & ((1 << bits) - 1)
                assert W[n, k] == float(cs.codebook[qv]) * float(s[n, b])


def test_per_row_scaling_special_case(impl):
    """Block size = K (per-row scaling, Sec. 3.1) is rank 1 with A = ones."""
    q, codes, C, B, _, _ = small_case(4, N=5, K=64, r=1)
    A = np.ones((1, 64), dtype=np.float32)
    W = impl.dequant(codes, C, B, A, 4)
    np.testing.assert_array_equal(W, C.astype(np.float64)[q] * B.astype(np.float64))


# ---------------------------------------------------------------------- Y
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_matmul_brute_force(impl, bits):
    q, codes, C, B, A, X = small_case(bits, N=5, K=32, r=2, M=3)
    Y = impl.matmul(X, codes, C, B, A, bits)
    assert Y.shape == (3, 5)
    for m in range(3):
        for n in range(5):
            terms = []
            for k in range(32):
                s = math.fsum(float(B[n, j]) * float(A[j, k]) for j in range(2))
                terms.append(float(X[m, k]) * float(C[q[n, k]]) * s)
            assert Y[m, n] == pytest.approx(math.fsum(terms), rel=1e-12, abs=1e-14)


def test_identity_activations_give_w_transposed(impl):
    q, codes, C, B, A, _ = small_case(3, N=7, K=64, r=5)
    Y = impl.matmul(np.eye(64, dtype=np.float32), codes, C, B, A, 3)
    np.testing.assert_allclose(Y, impl.dequant(codes, C, B, A, 3).T, rtol=0, atol=0)


def test_rank_one_closed_form(impl):
    """S = b a^T  =>  Y = ((X (.) a^T) C[q]^T) (.) b^T."""
    q, codes, C, B, A, X = small_case(4, N=9, K=96, r=1, M=4)
    Y = impl.matmul(X, codes, C, B, A, 4)
    Cq = C.astype(np.float64)[q]
    want = ((X.astype(np.float64) * A.astype(np.float64)[0][None, :]) @ Cq.T) * B.astype(np.float64)[:, 0][None, :]
    np.testing.assert_allclose(Y, want, rtol=1e-12, atol=1e-13)


def test_all_ones_table_is_plain_low_rank_product(impl):
    """C == 1  =>  W_hat = BA and Y = (X A^T) B^T."""
    _, codes, _, B, A, X = small_case(2, N=8, K=64, r=4, M=3)
    Y = impl.matmul(X, codes, np.ones(4, dtype=np.float32), B, A, 2)
    want = (X.astype(np.float64) @ A.astype(np.float64).T) @ B.astype(np.float64).T
    np.testing.assert_allclose(Y, want, rtol=1e-12, atol=1e-13)


def test_linearity(impl):
    _, codes, C, B, A, X = small_case(4, N=6, K=64, r=3, M=2)
    _, _, _, B2, A2, X2 = small_case(4, N=6, K=64, r=3, M=2, seed=2)
    f = lambda X_, B_, A_: impl.matmul(X_, codes, C, B_, A_, 4)
    # sums of fp32 arrays formed in fp64 then passed as fp32 would round; use exact dyadic scalings instead
    np.testing.assert_allclose(f(2 * X, B, A), 2 * f(X, B, A), rtol=1e-14)
    np.testing.assert_allclose(f(X, 0.5 * B, A), 0.5 * f(X, B, A), rtol=1e-14)
    np.testing.assert_allclose(f(X, B, -4 * A), -4 * f(X, B, A), rtol=1e-14)
    # additivity in X with fp32-exact sums: integers
    Xi = np.round(8 * X).astype(np.float32)
    Xj = np.round(8 * X2).astype(np.float32)
    np.testing.assert_allclose(f(Xi + Xj, B, A), f(Xi, B, A) + f(Xj, B, A), rtol=1e-12, atol=1e-12)
    # additivity in the factors through stacking ranks: [B B2][A; A2] = BA + B2A2
    Bs, As = np.concatenate([B, B2], 1), np.concatenate([A, A2], 0)
    np.testing.assert_allclose(f(X, Bs, As), f(X, B, A) + f(X, B2, A2), rtol=1e-12, atol=1e-12)


def test_row_subset_matches_full():
    cs = li.make_case("tiny")
    rows = np.array([0, 3, 511, 17])
    full = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    np.testing.assert_allclose(onp.matmul_rows(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4, rows),
                               full[:, rows], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(oc.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4, rows=rows),
                               full[:, rows], rtol=1e-12, atol=1e-15)


def test_two_oracles_agree_on_tiny_config():
    cs = li.make_case("tiny")
    Wn = onp.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    Wc = oc.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    assert onp.rel_fro(Wc, Wn) < 1e-14
    Yn = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    Yc = oc.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    assert onp.rel_fro(Yc, Yn) < 1e-13


# --------------------------------------------------------------- rank rule
def test_equivalent_rank_table7(golden_dir):
    rows = read_rank_table(os.path.join(golden_dir, "table7_ranks.txt"))
    assert len(rows) == 13
    for model, module, N, K, r128, r256 in rows:
        assert onp.equivalent_rank(N, K, 128) == r128, (model, module)
        assert onp.equivalent_rank(N, K, 256) == r256, (model, module)
    # the PEFT default point of Sec. 4.3: block 64 on 4096x4096 <-> rank 32
    assert onp.equivalent_rank(4096, 4096, 64) == 32


# ------------------------------------------------- the pins must have teeth
def _battery(impl):
    """A compact version of the pins above, raising AssertionError on any miss."""
    for bits, byts, codes in read_packed_golden(os.path.join(os.path.dirname(__file__), "golden", "packed_bytes.txt")):
        assert impl.unpack_codes(byts[None, :], codes.size, bits)[0].tolist() == codes.tolist()
    for bits in (2, 3, 4):
        q, codes, C, B, A, X = small_case(bits, N=4, K=32, r=3, M=2)
        W = impl.dequant(codes, C, B, A, bits)
        Y = impl.matmul(X, codes, C, B, A, bits)
        for n in range(4):
            w = [float(C[q[n, k]]) * math.fsum(float(B[n, j]) * float(A[j, k]) for j in range(3)) for k in range(32)]
            for k in range(32):
                assert W[n, k] == pytest.approx(w[k], rel=1e-13, abs=1e-300)
            for m in range(2):
                assert Y[m, n] == pytest.approx(math.fsum(float(X[m, k]) * w[k] for k in range(32)), rel=1e-12, abs=1e-14)


def _mutant(**repl):
    m = types.SimpleNamespace(unpack_codes=onp.unpack_codes, dequant=onp.dequant, matmul=onp.matmul)
    for k, v in repl.items():
        setattr(m, k, v)
    return m


def test_pins_catch_planted_mistakes():
    _battery(onp)     # the real oracle passes
    C64 = lambda c: np.asarray(c, dtype=np.float64)

    def unpack_high_first(codes, K, bits):      # wrong order inside a byte
        return onp.unpack_codes(codes, K, bits).reshape(codes.shape[0], -1, 8 // bits if bits != 3 else 8)[:, :, ::-1].reshape(codes.shape[0], K)

    def dequant_with(unpack=onp.unpack_codes, scale=onp.scale_matrix):
        def f(codes, codebook, B, A, bits):
            return C64(codebook)[unpack(codes, np.asarray(A).shape[1], bits)] * scale(B, A)
        return f

    def matmul_with(deq, xform=lambda Y: Y):
        return lambda X, codes, cb, B, A, bits: xform(C64(X) @ deq(codes, cb, B, A, bits).T)

    mutants = {
        "high bits first": _mutant(unpack_codes=unpack_high_first),
        "dropped last rank term": _mutant(dequant=dequant_with(scale=lambda B, A: onp.scale_matrix(B[:, :-1], A[:-1]))),
        "sign flip": _mutant(dequant=dequant_with(scale=lambda B, A: -onp.scale_matrix(B, A))),
        "A rows reversed": _mutant(dequant=dequant_with(scale=lambda B, A: onp.scale_matrix(B, A[::-1]))),
        "additive instead of multiplicative": _mutant(
            dequant=lambda codes, cb, B, A, bits: C64(cb)[onp.unpack_codes(codes, A.shape[1], bits)] + onp.scale_matrix(B, A)),
        "Y from codes off by one column": _mutant(
            matmul=matmul_with(lambda codes, cb, B, A, bits: np.roll(onp.dequant(codes, cb, B, A, bits), 1, axis=1))),
        "Y with squared table": _mutant(
            matmul=matmul_with(lambda codes, cb, B, A, bits: onp.dequant(codes, C64(cb) ** 2, B, A, bits))),
    }
    for name, m in mutants.items():
        with pytest.raises(AssertionError):
            _battery(m)
            pytest.fail(f"planted mistake not caught: {name}", pytrace=False)


# ------------------------------------------------------- input generator
def test_nf_codebook_properties():
    from scipy.stats import norm
    for bits in (2, 3, 4):
        C = li.nf_codebook(bits)
        n = 1 << bits
        assert C.shape == (n,) and C.dtype == np.float32
        assert C[0] == -1.0 and C[-1] == 1.0
        assert np.all(np.diff(C) > 0)
        np.testing.assert_allclose(C, -C[::-1], atol=1e-7)
        p = (np.arange(n) + 0.5) / n                 # second library routine for the quantile
        np.testing.assert_allclose(C, norm.ppf(p) / norm.ppf(p[-1]), atol=2e-7)
    assert li.nf_codebook(2)[2] == pytest.approx(0.276994, abs=1e-6)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927, 1e-3], dtype=np.float32)
    bits, vals = li.to_bf16(x)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert vals[0] == 1.0 and vals[1] == 1.0 and vals[2] == 1.015625
    assert np.all(np.abs(vals - x) <= np.abs(x) * 2.0 ** -8)
    np.testing.assert_array_equal(li.bf16_bits_to_f32(bits), vals)
    import torch
    np.testing.assert_array_equal(torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy(), vals)


# ------------------------------------------------------------------ the gate functions
def test_gate_functions_hand_values():
    """rel_fro and max_abs_over_rms carry every parity gate (W within relative Frobenius error 1e-3; Y
    within relative Frobenius error 5e-3 and |dY| <= 2e-2 rms(Y_oracle), as the benchmark spec words
    them), so they are pinned to values worked out by hand on a 2 x 2 case.
        want = [[3, 0], [0, 4]], got = [[3, 1], [1, 2]]:  got - want = [[0, 1], [1, -2]],
        |got - want|_F = sqrt(0 + 1 + 1 + 4) = sqrt(6),  |want|_F = sqrt(9 + 16) = 5,
        rms(want) = sqrt((9 + 0 + 0 + 16) / 4) = 2.5,  max|got - want| = 2."""
    want = np.array([[3.0, 0.0], [0.0, 4.0]])
    got = np.array([[3.0, 1.0], [1.0, 2.0]])
    assert onp.rel_fro(got, want) == pytest.approx(math.sqrt(6.0) / 5.0, rel=1e-15)
    assert onp.max_abs_over_rms(got, want) == pytest.approx(2.0 / 2.5, rel=1e-15)
    # not symmetric in its arguments: the reference is the second one
    assert onp.rel_fro(want, got) == pytest.approx(math.sqrt(6.0) / math.sqrt(9 + 1 + 1 + 4), rel=1e-15)
    assert onp.max_abs_over_rms(want, got) == pytest.approx(2.0 / math.sqrt(15.0 / 4.0), rel=1e-15)
    # equal arrays, a scaled copy, float32 input widened exactly
    assert onp.rel_fro(want, want) == 0.0 and onp.max_abs_over_rms(want, want) == 0.0
    assert onp.rel_fro(1.5 * want, want) == pytest.approx(0.5, rel=1e-15)
    assert onp.max_abs_over_rms(1.5 * want, want) == pytest.approx(0.5 * 4.0 / 2.5, rel=1e-15)
    assert onp.rel_fro(got.astype(np.float32), want.astype(np.float32)) == pytest.approx(math.sqrt(6.0) / 5.0, rel=1e-15)
    # a zero reference: the plain norm / the plain largest deviation (no division by zero)
    zero = np.zeros((2, 2))
    assert onp.rel_fro(got, zero) == pytest.approx(math.sqrt(9 + 1 + 1 + 4), rel=1e-15)
    assert onp.max_abs_over_rms(got, zero) == 3.0
    assert onp.rel_fro(zero, zero) == 0.0 and onp.max_abs_over_rms(zero, zero) == 0.0
    # a single wrong element among many: the element-wise gate sees it, the Frobenius gate barely
    big = np.ones((100, 100))
    off = big.copy()
    off[7, 9] = 1.5
    assert onp.max_abs_over_rms(off, big) == pytest.approx(0.5, rel=1e-15)
    assert onp.rel_fro(off, big) == pytest.approx(0.5 / 100.0, rel=1e-15)
    # not-a-number in the result must not pass a "<=" gate
    bad = got.copy()
    bad[0, 0] = np.nan
    assert not (onp.rel_fro(bad, want) <= 1.0) and not (onp.max_abs_over_rms(bad, want) <= 1.0)
