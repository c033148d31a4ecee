"""GPU parity of the backward entry points (lords_transpose_codes, lords_backward_input,
lords_backward_factors), called through the C ABI, against the fp64 oracle on the same seeded inputs.

Gates: transposed codes bit-exact; dX as Y of lords_matmul (it is the same product, of the transposed
layer): relative Frobenius error <= 5e-3, max |d| <= 2e-2 * rms.  dB and dA: relative Frobenius error
<= 5e-3; element by element |d| <= 2e-2 * rms + 2^-7 |want|.  (G is summed in fp32; P = level * G and the
factor it meets are each rounded once to bf16, 2^-9 relative each, so every term of the second sum
carries up to 2^-8 relative error; where that sum has few terms, e.g. 16 rows, the errors do not
average out and an element can be off by that much of its own size: hence the 2^-7 |want| term, twice
the worst case of one term.)
"""
import sys

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp

pytestmark = pytest.mark.gpu

TOL, MAX_TOL = 5e-3, 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def check(got, want, what):
    rf, mx = onp.rel_fro(got, want), onp.max_abs_over_rms(got, want)
    say(f"   {what}: rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(got).all(), what
    assert rf <= TOL, (what, rf)
    assert mx <= MAX_TOL, (what, mx)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(32, 32), (64, 96), (96, 544), (128, 4096), (4096, 256), (320, 288)])
def test_transpose_codes_bit_exact(gpu, bits, N, K):
    import torch
    import paper_2601_22716_amd as L
    say(f"transpose_codes bits={bits} N={N} K={K}")
    cs = li.make_case("tiny", N=N, K=K, bits=bits, r=1, seed=51)
    codes = torch.from_numpy(cs.codes.copy()).cuda()
    out = torch.full((K, N * bits // 8), 0xA5, dtype=torch.uint8, device="cuda")
    L.lords_transpose_codes(codes, out, N, K, bits)
    torch.cuda.synchronize()
    q = onp.unpack_codes(cs.codes, K, bits)
    np.testing.assert_array_equal(out.cpu().numpy(), onp.pack_codes(q.T.copy(), bits))


def check_grad(got, want, what):
    rf = onp.rel_fro(got, want)
    rms = float(np.sqrt(np.mean(np.asarray(want, dtype=np.float64) ** 2)))
    worst = float((np.abs(got - want) / (MAX_TOL * rms + 2.0 ** -7 * np.abs(want) + 1e-30)).max())
    say(f"   {what}: rel_fro={rf:.2e} worst |d|/bound={worst:.2f}")
    assert np.isfinite(got).all(), what
    assert rf <= TOL, (what, rf)
    assert worst <= 1.0, (what, worst)


def upload_grad(gpu, M, N, seed):
    bits16, vals = li.make_output_grad(M, N, seed)
    return gpu.bf16_tensor(bits16), vals


BW_SHAPES = [
    # N, K, r, M
    (32, 32, 1, 1),
    (64, 160, 5, 3),
    (512, 256, 4, 16),
    (96, 544, 32, 40),
    (1056, 288, 33, 7),
    (2080, 320, 64, 300),
    (4128, 128, 24, 1),
]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r,M", BW_SHAPES)
def test_backward_input_parity(gpu, bits, fdt, N, K, r, M):
    import torch
    import paper_2601_22716_amd as L
    say(f"backward_input bits={bits} factors={fdt} N={N} K={K} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=52, signed_factors=True)
    d = gpu.DeviceCase(cs)
    dY, dY32 = upload_grad(gpu, M, N, 52)
    codes_t = torch.empty((K, N * bits // 8), dtype=torch.uint8, device="cuda")
    L.lords_transpose_codes(d.codes, codes_t, N, K, bits)
    dX = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_input(dY, codes_t, d.codebook, d.B, d.A, dX, M, N, K, r, bits)
    torch.cuda.synchronize()
    want = onp.backward_input(dY32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check(dX.cpu().numpy(), want, "dX")


FG_SHAPES = [
    # N, K, r, M: ragged token counts, rows not a multiple of the 256-row tile, columns not a multiple of 128
    (8, 32, 1, 1),
    (40, 160, 5, 3),
    (512, 256, 4, 64),
    (264, 544, 32, 100),
    (1000, 288, 33, 130),
    (300 - 4, 320, 64, 257),
    (4096, 128, 24, 17),
    (16, 4128, 48, 70),
]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r,M", FG_SHAPES)
def test_backward_factors_parity(gpu, bits, fdt, N, K, r, M):
    import torch
    import paper_2601_22716_amd as L
    say(f"backward_factors bits={bits} factors={fdt} N={N} K={K} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=53, signed_factors=True)
    d = gpu.DeviceCase(cs)
    dY, dY32 = upload_grad(gpu, M, N, 53)
    dB = torch.full((N, r), float("nan"), dtype=torch.float32, device="cuda")
    dA = torch.full((r, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, M, N, K, r, bits)
    torch.cuda.synchronize()
    wB, wA = onp.backward_factors(dY32, cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check_grad(dB.cpu().numpy(), wB, "dB")
    check_grad(dA.cpu().numpy(), wA, "dA")
    # run-to-run identical
    dB2, dA2 = torch.empty_like(dB), torch.empty_like(dA)
    L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB2, dA2, M, N, K, r, bits)
    torch.cuda.synchronize()
    assert torch.equal(dB, dB2) and torch.equal(dA, dA2)


def test_backward_factors_blockwise_case(gpu):
    """A = block indicator (Sec. 3.1): dB[n][j] is the sum of level * G over block j of row n."""
    import torch
    import paper_2601_22716_amd as L
    N, K, bits, group, M = 96, 256, 4, 64, 50
    cs = li.make_blockwise_case(N, K, bits, group, M=M, seed=54)
    d = gpu.DeviceCase(cs)
    dY, dY32 = upload_grad(gpu, M, N, 54)
    r = K // group
    dB = torch.empty((N, r), dtype=torch.float32, device="cuda")
    dA = torch.empty((r, K), dtype=torch.float32, device="cuda")
    L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, M, N, K, r, bits)
    torch.cuda.synchronize()
    G = dY32.astype(np.float64).T @ cs.X_f32.astype(np.float64)
    P = cs.codebook.astype(np.float64)[onp.unpack_codes(cs.codes, K, bits)] * G
    check_grad(dB.cpu().numpy(), P.reshape(N, r, group).sum(axis=2), "dB, block sums")


def test_backward_unsupported_and_empty(gpu):
    import torch
    import paper_2601_22716_amd as L
    cs = li.make_case("tiny", M=2, N=36, K=64, bits=4, r=4, factor_dtype="bf16", seed=55)
    d = gpu.DeviceCase(cs)
    dY, _ = upload_grad(gpu, 2, 36, 55)
    dB = torch.empty((36, 4), dtype=torch.float32, device="cuda")
    dA = torch.empty((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LordsError) as e:                  # N not a multiple of 8
        L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, 2, 36, 64, 4, 4)
    assert e.value.status == 7
    # no tokens: zero gradients
    cs = li.make_case("tiny", M=1, N=40, K=64, bits=4, r=4, factor_dtype="bf16", seed=56)
    d = gpu.DeviceCase(cs)
    dB = torch.full((40, 4), float("nan"), dtype=torch.float32, device="cuda")
    dA = torch.full((4, 64), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_factors(d.X, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, 0, 40, 64, 4, 4)
    torch.cuda.synchronize()
    assert float(dB.abs().max()) == 0.0 and float(dA.abs().max()) == 0.0


@pytest.mark.parametrize("name,M", [("gateup_4b", 2048), ("qproj_4b", 512), ("down_3b", 256)])
def test_full_size_backward_sampled(gpu, name, M):
    """Full layer shapes: sampled columns of dX, rows of dB and columns of dA against the oracle's
    restricted forms."""
    import torch
    import paper_2601_22716_amd as L
    cfg = li.CONFIGS[name]
    N, K, r, bits = cfg.N, cfg.K, cfg.r, cfg.bits
    say(f"full-size backward {name} M={M}")
    cs = li.make_case(name, M=M, seed=57, signed_factors=True)
    d = gpu.DeviceCase(cs)
    dY, dY32 = upload_grad(gpu, M, N, 57)
    codes_t = torch.empty((K, N * bits // 8), dtype=torch.uint8, device="cuda")
    L.lords_transpose_codes(d.codes, codes_t, N, K, bits)
    dX = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_input(dY, codes_t, d.codebook, d.B, d.A, dX, M, N, K, r, bits)
    dB = torch.full((N, r), float("nan"), dtype=torch.float32, device="cuda")
    dA = torch.full((r, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, M, N, K, r, bits)
    torch.cuda.synchronize()
    dXh, dBh, dAh = dX.cpu().numpy(), dB.cpu().numpy(), dA.cpu().numpy()
    assert np.isfinite(dXh).all() and np.isfinite(dBh).all() and np.isfinite(dAh).all()
    rng = np.random.default_rng(570)
    cols = np.unique(np.concatenate([[0, K - 1], rng.integers(0, K, 62)]))
    rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 62)]))
    toks = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 30)]))
    check(dXh[np.ix_(toks, cols)],
          onp.backward_input_cols(dY32[toks], cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits, cols), "dX sample")
    check_grad(dBh[rows], onp.backward_factors_rows(dY32, cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits, rows),
          "dB sample")
    check_grad(dAh[:, cols], onp.backward_factors_cols(dY32, cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits, cols),
          "dA sample")
