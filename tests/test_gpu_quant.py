"""GPU parity of the quantisation side through the C ABI: lords_quantize (Alg. 1 step 2.1) and
lords_block_init (block-wise scale of step 1 as factors).  The level index is an integer decided by
floating point, so the oracle takes the decision in the same stated fp32 operations
(oracle/lords_oracle.c) and the comparison is bit for bit; the fp64 statement of the definition
bounds how far from optimal any index may be."""
from __future__ import annotations

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp
from oracle import lords_oracle_c as oc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2601_22716_amd as L
    L.library()
    return types_ns(torch, L)


def types_ns(torch, L):
    import types
    return types.SimpleNamespace(torch=torch, L=L)


def say(msg):
    print(msg, flush=True)


def weights(seed, N, K, dtype):
    """Weights with the heavy tails of a real layer: N(0, 0.02) plus a few outliers."""
    g = np.random.default_rng([seed, 31])
    W = (0.02 * g.standard_normal((N, K))).astype(np.float32)
    out = g.random((N, K)) < 0.002
    W[out] *= 8.0
    if dtype == "bf16":
        bits, W = li.to_bf16(W)
        return bits, W
    return None, W


def upload(gpu, bits_u16, f32):
    if bits_u16 is not None:
        return gpu.L.bf16_from_bits(bits_u16)
    return gpu.torch.from_numpy(np.ascontiguousarray(f32)).cuda()


def run_quantize(gpu, Wbits, W, codebook, Bt, At, N, K, r, bits):
    t = gpu.torch
    codes = t.full((N, K * bits // 8), 0xAA, dtype=t.uint8, device="cuda")
    gpu.L.lords_quantize(upload(gpu, Wbits, W), t.from_numpy(codebook.copy()).cuda(), Bt, At, codes, N, K, r, bits)
    t.cuda.synchronize()
    return codes.cpu().numpy()


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("wdt", ["f32", "bf16"])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r", [(1, 32, 1), (70, 160, 5), (300, 4128, 32)])
def test_quantize_matches_fp32_oracle_bit_for_bit(gpu, bits, wdt, fdt, N, K, r):
    say(f"quantize bits={bits} W={wdt} factors={fdt} N={N} K={K} r={r}")
    cs = li.make_case("tiny", N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=17, signed_factors=True)
    Wbits, W = weights(3, N, K, wdt)
    if fdt == "bf16":
        Bt, At = gpu.L.bf16_from_bits(cs.B_bf16), gpu.L.bf16_from_bits(cs.A_bf16)
    else:
        Bt, At = gpu.torch.from_numpy(cs.B_f32.copy()).cuda(), gpu.torch.from_numpy(cs.A_f32.copy()).cuda()
    got = run_quantize(gpu, Wbits, W, cs.codebook, Bt, At, N, K, r, bits)
    want_q = oc.quantize_f32(W, cs.codebook, cs.B_f32, cs.A_f32, bits)
    np.testing.assert_array_equal(got, onp.pack_codes(want_q, bits))
    # and against the definition in fp64: never worse than the best level by more than rounding
    q = onp.unpack_codes(got, K, bits)
    S = onp.scale_matrix(cs.B_f32, cs.A_f32)
    C = cs.codebook.astype(np.float64)
    err = (S * C[q] - W) ** 2
    best = ((S[:, :, None] * C - W[:, :, None].astype(np.float64)) ** 2).min(axis=2)
    assert np.all(err <= best + 1e-5 * (np.abs(S) * np.abs(C).max() + np.abs(W)) ** 2)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_inverts_dequant(gpu, bits):
    """codes -> lords_dequant -> lords_quantize gives the codes back (distinct levels, non-zero scales)."""
    say(f"quantize(dequant(codes)) bits={bits}")
    from tests import gpu_util
    cs = li.make_case("tiny", N=257, K=544, bits=bits, r=12, factor_dtype="f32", seed=5, signed_factors=True)
    d = gpu_util.DeviceCase(cs)
    W = d.dequant()                                         # fp32
    got = run_quantize(gpu, None, W, cs.codebook, d.B, d.A, cs.N, cs.K, cs.r, bits)
    np.testing.assert_array_equal(got, cs.codes)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("wdt", ["f32", "bf16"])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r", [(3, 32, 1), (65, 640, 5), (128, 4096, 32), (40, 96, 96),
                                   # block sizes 4, 8 and 256 (one to sixty-four lanes per block), a ragged last wave;
                                   # 448 does not divide 256: the one-wave-per-block kernel
                                   (17, 64, 16), (5, 64, 8), (33, 1024, 4), (9, 1344, 3), (1000, 2048, 64)])
def test_block_init_bit_exact(gpu, bits, wdt, fdt, N, K, r):
    say(f"block_init bits={bits} W={wdt} factors={fdt} N={N} K={K} r={r}")
    t = gpu.torch
    Wbits, W = weights(9, N, K, wdt)
    C = li.nf_codebook(bits)
    dt = t.float32 if fdt == "f32" else t.bfloat16
    B = t.full((N, r), float("nan"), dtype=dt, device="cuda")
    A = t.full((r, K), float("nan"), dtype=dt, device="cuda")
    gpu.L.lords_block_init(upload(gpu, Wbits, W), t.from_numpy(C.copy()).cuda(), B, A, N, K, r, bits)
    t.cuda.synchronize()
    B32, A32 = oc.block_init_f32(W, C, r, bits)
    if fdt == "bf16":
        B32, A32 = li.to_bf16(B32)[1], li.to_bf16(A32)[1]
    np.testing.assert_array_equal(B.float().cpu().numpy(), B32)
    np.testing.assert_array_equal(A.float().cpu().numpy(), A32)


def test_blockwise_round_trip_on_a_layer_shape(gpu):
    """Whole chain on a full row range of a layer: block_init -> quantize -> dequant; the error of every
    weight is at most half the widest table gap times its block scale (Sec. 3.1, nearest-level rounding)."""
    from tests import gpu_util
    t, L = gpu.torch, gpu.L
    N, K, r, bits = 1024, 4096, 32, 4
    say(f"block-wise round trip N={N} K={K} r={r}")
    _, W = weights(12, N, K, "f32")
    C = li.nf_codebook(bits)
    Wd, Cd = t.from_numpy(W).cuda(), t.from_numpy(C.copy()).cuda()
    B = t.empty((N, r), dtype=t.float32, device="cuda"); A = t.empty((r, K), dtype=t.float32, device="cuda")
    codes = t.empty((N, K * bits // 8), dtype=t.uint8, device="cuda")
    What = t.empty((N, K), dtype=t.float32, device="cuda")
    L.lords_block_init(Wd, Cd, B, A, N, K, r, bits)
    L.lords_quantize(Wd, Cd, B, A, codes, N, K, r, bits)
    L.lords_dequant(codes, Cd, B, A, What, N, K, r, bits)
    t.cuda.synchronize()
    S = np.repeat(B.cpu().numpy().astype(np.float64), K // r, axis=1)
    gap = float(np.max(np.diff(C.astype(np.float64))))
    assert np.all(np.abs(What.cpu().numpy().astype(np.float64) - W) <= 0.5 * gap * S * (1 + 1e-5) + 1e-12)
    # same codes as the oracle on sampled rows
    rows = np.array([0, 1, 511, 1023])
    want = oc.quantize_f32(W[rows], C, B.cpu().numpy()[rows], A.cpu().numpy(), bits)
    np.testing.assert_array_equal(codes.cpu().numpy()[rows], onp.pack_codes(want, bits))
