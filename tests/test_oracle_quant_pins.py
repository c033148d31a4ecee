"""Pins of the quantisation side of the oracle (Alg. 1 step 2.1, the block-wise scale of step 1, the
packer) against things other than itself: hand-derived bytes, an independent packer, scalar brute
force, the textbook nearest-level rounding of Sec. 3.1, exact recovery of a quantised matrix, and
planted mistakes.  No GPU."""
from __future__ import annotations

import os
import types

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp
from oracle import lords_oracle_c as oc
from tests.helpers import pack_codes_py, read_packed_golden

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def rng(seed):
    return np.random.default_rng([seed, 77])


# ------------------------------------------------------------------ packer
@pytest.mark.parametrize("impl", [onp.pack_codes, oc.pack_codes], ids=["numpy", "c"])
def test_pack_hand_bytes(impl):
    for bits, byts, codes in read_packed_golden(os.path.join(GOLDEN, "packed_bytes.txt")):
        np.testing.assert_array_equal(impl(codes[None, :], bits)[0], byts)


@pytest.mark.parametrize("impl", [onp.pack_codes, oc.pack_codes], ids=["numpy", "c"])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_matches_bigint_packer_and_inverts_unpack(impl, bits):
    q = rng(bits).integers(0, 1 << bits, size=(7, 96), dtype=np.uint8)
    packed = impl(q, bits)
    np.testing.assert_array_equal(packed, pack_codes_py(q, bits))
    np.testing.assert_array_equal(onp.unpack_codes(packed, 96, bits), q)


# ------------------------------------------------------------------ quantise
def random_problem(seed, N, K, r, bits, signed=True):
    g = rng(seed)
    B = (g.standard_normal((N, r)) if signed else g.uniform(0.5, 1.5, (N, r))).astype(np.float32)
    A = (g.standard_normal((r, K)) if signed else g.uniform(0.5, 1.5, (r, K))).astype(np.float32)
    W = g.standard_normal((N, K)).astype(np.float32)
    return W, li.nf_codebook(bits), B, A


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_brute_force(bits):
    W, C, B, A = random_problem(1, 5, 32, 3, bits)
    got = onp.quantize(W, C, B, A)
    for n in range(5):
        for k in range(32):
            s = sum(float(B[n, j]) * float(A[j, k]) for j in range(3))
            errs = [(s * float(C[i]) - float(W[n, k])) ** 2 for i in range(1 << bits)]
            assert got[n, k] == errs.index(min(errs))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_is_nearest_level_rounding_of_w_over_s(bits):
    """Sec. 3.1: with one positive scale per element the quantiser is Round(W / S), the nearest
    level of the table; for a sorted table that is a search among the mid-points."""
    W, C, B, A = random_problem(2, 9, 64, 4, bits, signed=False)
    S = onp.scale_matrix(B, A)
    mids = (C[1:].astype(np.float64) + C[:-1].astype(np.float64)) / 2
    want = np.searchsorted(mids, W.astype(np.float64) / S)
    np.testing.assert_array_equal(onp.quantize(W, C, B, A), want)
    # a negative scale mirrors the table
    np.testing.assert_array_equal(onp.quantize(W, C, -B, A), np.searchsorted(mids, W.astype(np.float64) / -S))


@pytest.mark.parametrize("impl", ["exact", "f32"])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_recovers_a_quantised_matrix(impl, bits):
    """W = C[q] (.) S is reproduced exactly: its own codes have zero error, every other level a
    positive one (distinct levels, non-zero scales)."""
    cs = li.make_case("tiny", N=40, K=96, bits=bits, r=5, factor_dtype="f32", seed=3, signed_factors=True)
    q = onp.unpack_codes(cs.codes, cs.K, bits)
    W = onp.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    if impl == "exact":
        got = onp.quantize(W, cs.codebook, cs.B_f32, cs.A_f32)
    else:
        got = oc.quantize_f32(W.astype(np.float32), cs.codebook, cs.B_f32, cs.A_f32, bits)
    np.testing.assert_array_equal(got, q)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_f32_agrees_with_fp64_except_at_near_ties(bits):
    W, C, B, A = random_problem(4, 33, 160, 7, bits)
    q64, margin = onp.quantize(W, C, B, A, with_margin=True)
    q32 = oc.quantize_f32(W, C, B, A, bits)
    differ = q64 != q32
    S = onp.scale_matrix(B, A)
    scale = (np.abs(S) * float(np.max(np.abs(C))) + np.abs(W)) ** 2
    assert np.all(margin[differ] <= 1e-5 * scale[differ])
    assert differ.mean() < 1e-3
    # and where they differ, the fp32 choice is (nearly) as good
    e = lambda q: (S * C[q].astype(np.float64) - W) ** 2
    assert np.all(e(q32) <= e(q64) + 1e-5 * scale)


def test_quantize_zero_scale_and_ties_take_the_lowest_index():
    C = li.int_codebook(2)                 # [-2, -1, 0, 1]
    B = np.zeros((1, 1), np.float32); A = np.ones((1, 32), np.float32)
    W = np.full((1, 32), 0.3, np.float32)
    assert np.all(onp.quantize(W, C, B, A) == 0) and np.all(oc.quantize_f32(W, C, B, A, 2) == 0)
    # exactly half way between levels -1 and 0 (indices 1, 2): the lower index wins
    B[:] = 1.0
    W[:] = -0.5
    assert np.all(onp.quantize(W, C, B, A) == 1) and np.all(oc.quantize_f32(W, C, B, A, 2) == 1)


# ------------------------------------------------------------------ block-wise initialisation
@pytest.mark.parametrize("bits", [2, 4])
def test_block_init_is_absmax_scaling(bits):
    g = rng(5)
    W = g.standard_normal((6, 128)).astype(np.float32)
    C = li.nf_codebook(bits)
    r, grp = 4, 32
    B, A = onp.block_init(W, C, r)
    S = onp.scale_matrix(B, A)
    cmax = float(np.max(np.abs(C)))
    for n in range(6):
        for j in range(r):
            blk = np.abs(W[n, j * grp:(j + 1) * grp].astype(np.float64))
            assert np.all(S[n, j * grp:(j + 1) * grp] == blk.max() / cmax)   # piecewise constant, Sec. 3.1
    # every normalised weight lies inside the table's range and each block touches its edge
    ratio = np.abs(W / S)
    assert ratio.max() <= cmax * (1 + 1e-12)
    assert np.allclose(ratio.reshape(6, r, grp).max(axis=2), cmax)
    # the fp32 statement agrees to rounding, and its A is the same indicator
    B32, A32 = oc.block_init_f32(W, C, r, bits)
    np.testing.assert_array_equal(A32, A.astype(np.float32))
    np.testing.assert_allclose(B32, B, rtol=1e-6)
    assert np.linalg.matrix_rank(S) <= r


def test_blockwise_quantise_dequantise_error_bound():
    """Block-wise quantisation through the factor form: error of each weight is at most half the
    widest gap of the table times its block scale (nearest-level rounding inside the range)."""
    W = rng(6).standard_normal((16, 256)).astype(np.float32)
    C = li.nf_codebook(4)
    B, A = onp.block_init(W, C, 8)
    q = onp.quantize(W, C, B, A)
    What = onp.dequant(onp.pack_codes(q, 4), C, B, A, 4)
    S = onp.scale_matrix(B, A)
    assert np.all(np.abs(What - W) <= 0.5 * np.max(np.diff(C.astype(np.float64))) * S + 1e-12)


# ------------------------------------------------------------------ planted mistakes
def test_quant_pins_catch_planted_mistakes():
    W, C, B, A = random_problem(7, 9, 64, 4, 3, signed=False)
    S = onp.scale_matrix(B, A)
    mids = (C[1:].astype(np.float64) + C[:-1].astype(np.float64)) / 2
    want = np.searchsorted(mids, W.astype(np.float64) / S)
    mutants = {
        "argmax": lambda: np.argmax((S[:, :, None] * C - W[:, :, None].astype(np.float64)) ** 2, axis=2),
        "scale on the wrong side": lambda: np.argmin((C[None, None, :] - S[:, :, None] * W[:, :, None]) ** 2, axis=2),
        "transposed factors": lambda: onp.quantize(W, C, B[:, ::-1], A),
        "absolute instead of signed": lambda: np.argmin((S[:, :, None] * np.abs(C) - W[:, :, None]) ** 2, axis=2),
    }
    for name, f in mutants.items():
        assert not np.array_equal(f(), want), name
