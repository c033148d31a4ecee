"""lords_repack (slab-tile layout of the codes) and lords_matmul_repacked, through the C ABI: the tiled
buffer equals the oracle's byte for byte; products on the tiled matrix are inside the gates against
the oracle and, where the same kernel runs with the same plan, bit-identical to lords_matmul."""
import sys

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp

pytestmark = pytest.mark.gpu

Y_TOL, Y_MAX_TOL = 5e-3, 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def tiled_codes(L, d, N, K, bits):
    import torch
    t = torch.full((L.lords_repack_bytes(N, K, bits),), 0xA5, dtype=torch.uint8, device="cuda")
    L.lords_repack(d.codes, t, N, K, bits)
    torch.cuda.synchronize()
    return t


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(1, 32), (16, 128), (17, 160), (37, 288), (300, 1056), (1000, 2592)])
def test_repack_bit_exact(gpu, bits, N, K):
    import paper_2601_22716_amd as L
    say(f"repack bits={bits} N={N} K={K}")
    cs = li.make_case("tiny", M=1, N=N, K=K, bits=bits, r=8, factor_dtype="bf16", seed=N + K + bits)
    d = gpu.DeviceCase(cs)
    got = tiled_codes(L, d, N, K, bits).cpu().numpy()
    want = onp.repack_codes(cs.codes, N, K, bits)
    assert got.size == want.size == L.lords_repack_bytes(N, K, bits)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("bits,N,K,r", [(4, 1000, 2592, 32), (3, 520, 1056, 20), (2, 333, 4128, 48), (4, 257, 544, 64), (2, 640, 8192, 100)])
@pytest.mark.parametrize("M", [1, 2, 5, 16, 40, 300])
def test_matmul_repacked_parity(gpu, bits, N, K, r, M):
    import torch
    import paper_2601_22716_amd as L
    say(f"repacked matmul bits={bits} N={N} K={K} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=41, signed_factors=True)
    d = gpu.DeviceCase(cs)
    t = tiled_codes(L, d, N, K, bits)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    if r > 64 and M == 1:
        # one token at ranks above 64 belongs to a fallback kernel that reads canonical rows only
        with pytest.raises(L.LordsError) as e:
            L.lords_matmul_repacked(d.X, t, d.codebook, d.B, d.A, Y, M, N, K, r, bits)
        assert e.value.status == 7
        return
    L.lords_matmul_repacked(d.X, t, d.codebook, d.B, d.A, Y, M, N, K, r, bits)
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    rf, mx = onp.rel_fro(got, want), onp.max_abs_over_rms(got, want)
    say(f"   rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(got).all()
    assert rf <= Y_TOL and mx <= Y_MAX_TOL, (rf, mx)
    # from three tokens on the same kernel runs with the same plan on either layout: same sums, same order
    if M >= 3:
        np.testing.assert_array_equal(got, d.matmul(M=M))


def test_matmul_repacked_full_size_sampled(gpu):
    import torch
    import paper_2601_22716_amd as L
    from oracle import lords_oracle_c as oc
    for name, M in (("gateup_4b", 1), ("down_3b", 1), ("l70b_2b", 1), ("gateup_4b", 16), ("gateup_4b", 300)):
        cfg = li.CONFIGS[name]
        say(f"repacked full size {name} M={M}")
        cs = li.make_case(name, M=M, seed=17)
        d = gpu.DeviceCase(cs)
        t = tiled_codes(L, d, cfg.N, cfg.K, cfg.bits)
        Y = torch.full((M, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
        L.lords_matmul_repacked(d.X, t, d.codebook, d.B, d.A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)
        torch.cuda.synchronize()
        rows = np.unique(np.concatenate([[0, 1, 15, 16, cfg.N - 17, cfg.N - 1], np.random.default_rng(3).integers(0, cfg.N, 150)]))
        want = oc.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, cfg.bits, rows=rows)
        got = Y.cpu().numpy()
        assert np.isfinite(got).all()
        rf, mx = onp.rel_fro(got[:, rows], want), onp.max_abs_over_rms(got[:, rows], want)
        say(f"   rel_fro={rf:.2e} max/rms={mx:.2e}")
        assert rf <= Y_TOL and mx <= Y_MAX_TOL, (name, M, rf, mx)


def test_repacked_rejects_what_the_fast_kernels_do_not_take(gpu):
    import torch
    import paper_2601_22716_amd as L
    cs = li.make_case("tiny")                                 # fp32 factors: fallback kernels, canonical rows only
    d = gpu.DeviceCase(cs)
    t = tiled_codes(L, d, cs.N, cs.K, cs.bits)
    Y = torch.empty((cs.M, cs.N), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LordsError) as e:
        L.lords_matmul_repacked(d.X, t, d.codebook, d.B, d.A, Y, cs.M, cs.N, cs.K, cs.r, cs.bits)
    assert e.value.status == 7
