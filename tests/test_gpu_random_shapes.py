"""GPU parity on a fixed list of pseudo-randomly drawn VALID shapes (seeded: the same list every run),
for every multiplying entry point, against the fp64 oracle.  The hand-picked shapes of the other test
files aim at known tile edges; these are meant to land between them.
"""
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

def same_as_single(Y, single, M, what):
    """A batched call against the single-matrix call on the same inputs.  From three tokens on both
    run the same kernel and sum every row in the same order: bit-identical.  With one or two tokens
    the single-matrix call takes the regrouped one-/two-token kernel and the batched call the
    shared-launch kernels: two roundings of the same sums, each inside the gates against the oracle,
    so they may differ by twice the element-wise gate at most."""
    if M > 2:
        np.testing.assert_array_equal(Y, single, err_msg=f"{what}: batched and single-matrix calls differ")
    elif single.size >= 16:                  # (the rms of a handful of outputs is no scale: those are judged against the oracle only)
        rms = float(np.sqrt(np.mean(single.astype(np.float64) ** 2))) + 1e-30
        worst = float(np.abs(Y.astype(np.float64) - single).max()) / rms
        assert worst <= 2 * Y_MAX_TOL, (what, worst)



@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def draw(i):
    """Shape number i: N, K, r, M, bits, factor dtype."""
    g = np.random.default_rng([2601, 22716, i])
    bits = int(g.choice([2, 3, 4]))
    K = 32 * int(g.integers(1, 70))
    N = int(g.integers(1, 700))
    r = int(g.choice([1, 3, 8, 16, 24, 32, 40, 48, 64, 80, 128]))
    M = int(g.choice([1, 2, 3, 7, 16, 17, 31, 33, 64, 100, 129, 260]))
    fdt = "bf16" if g.random() < 0.7 else "f32"
    return N, K, r, M, bits, fdt


def check(Y, want, what, floor_rms=None):
    rf, mx = onp.rel_fro(Y, want), onp.max_abs_over_rms(Y, want)
    say(f"   {what}: rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(Y).all(), what
    assert rf <= Y_TOL, (what, rf)
    assert mx <= Y_MAX_TOL, (what, mx)


@pytest.mark.parametrize("i", range(48))
def test_matmul_random_shape(gpu, i):
    N, K, r, M, bits, fdt = draw(i)
    say(f"matmul #{i}: N={N} K={K} r={r} M={M} bits={bits} factors={fdt}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=700 + i, signed_factors=True)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    d = gpu.DeviceCase(cs)
    check(d.matmul(), want, "automatic path")
    import paper_2601_22716_amd as L
    check(d.matmul(path=L.LORDS_PATH_DECODE), want, "decode kernels")
    check(d.matmul(path=L.LORDS_PATH_PREFILL), want, "GEMM kernels")


@pytest.mark.parametrize("i", range(16))
def test_shared_input_random_shape(gpu, i):
    import torch
    import paper_2601_22716_amd as L
    g = np.random.default_rng([2601, 22716, 1000 + i])
    _, K, r, M, bits, _ = draw(100 + i)
    r = min(r, 64)
    M = int(g.choice([1, 1, 2, 5, 16, 20]))
    Ns = [int(n) for n in g.integers(1, 400, size=int(g.integers(2, 9)))]
    say(f"batched #{i}: Ns={Ns} K={K} r={r} M={M} bits={bits}")
    cases = [li.make_case("tiny", M=M, N=n, K=K, bits=bits, r=r, factor_dtype="bf16", seed=800 + 16 * i + j,
                          signed_factors=True) for j, n in enumerate(Ns)]
    dev = [gpu.DeviceCase(c) for c in cases]
    Ys = [torch.full((M, n), float("nan"), dtype=torch.float32, device="cuda") for n in Ns]
    L.lords_matmul_batched(dev[0].X, [d.codes for d in dev], dev[0].codebook, [d.B for d in dev], [d.A for d in dev], Ys,
                           Ns, M, K, r, bits)
    torch.cuda.synchronize()
    want = onp.matmul_batched(cases[0].X_f32, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, bits)
    for l, (Y, w) in enumerate(zip(Ys, want)):
        got = Y.cpu().numpy()
        same_as_single(got, dev[l].matmul(X=dev[0].X, M=M), M, f"matrix {l}")
        check(got, w, f"matrix {l}")


@pytest.mark.parametrize("i", range(16))
def test_backward_random_shape(gpu, i):
    import torch
    import paper_2601_22716_amd as L
    N, K, r, M, bits, fdt = draw(200 + i)
    N = 32 * max(1, N // 32)                                  # the transposed codes need whole groups of 32 rows
    r = min(r, 64)
    say(f"backward #{i}: N={N} K={K} r={r} M={M} bits={bits} factors={fdt}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=900 + i, signed_factors=True)
    d = gpu.DeviceCase(cs)
    dYb, dY32 = li.make_output_grad(M, N, 900 + i)
    dY = gpu.bf16_tensor(dYb)
    codes_t = torch.empty((K, N * bits // 8), dtype=torch.uint8, device="cuda")
    L.lords_transpose_codes(d.codes, codes_t, N, K, bits)
    dX = torch.full((M, K), float("nan"), dtype=torch.float32, device="cuda")
    dB = torch.full((N, r), float("nan"), dtype=torch.float32, device="cuda")
    dA = torch.full((r, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_backward_input(dY, codes_t, d.codebook, d.B, d.A, dX, M, N, K, r, bits)
    L.lords_backward_factors(dY, d.X, d.codes, d.codebook, d.B, d.A, dB, dA, M, N, K, r, bits)
    torch.cuda.synchronize()
    check(dX.cpu().numpy(), onp.backward_input(dY32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits), "dX")
    wB, wA = onp.backward_factors(dY32, cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    for got, want, what in ((dB.cpu().numpy(), wB, "dB"), (dA.cpu().numpy(), wA, "dA")):
        rms = float(np.sqrt(np.mean(want ** 2)))
        worst = float((np.abs(got - want) / (Y_MAX_TOL * rms + 2.0 ** -7 * np.abs(want) + 1e-30)).max())
        rf = onp.rel_fro(got, want)
        say(f"   {what}: rel_fro={rf:.2e} worst |d|/bound={worst:.2f}")
        assert np.isfinite(got).all()
        assert worst <= 1.0, (what, worst)
        if want.size >= 64:
            assert rf <= Y_TOL, (what, rf)
