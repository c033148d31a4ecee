"""GPU parity of a mixed-precision stack (Sec. 4.2, ultra-low-bit setting): the code width of each
layer comes from lords_mixed_schedule, every layer then runs through the ordinary entry points
with its own width, and every layer's output is compared with the fp64 oracle at that width.

Gates as for lords_matmul: relative Frobenius error <= 5e-3 and max |d| <= 2e-2 * rms(oracle);
H = silu(G) * U as in the shared-input tests.
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


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def check(Y, want, what):
    rf, mx = onp.rel_fro(Y, want), onp.max_abs_over_rms(Y, want)
    say(f"   {what}: rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(Y).all(), what
    assert rf <= Y_TOL, (what, rf)
    assert mx <= Y_MAX_TOL, (what, mx)


@pytest.mark.parametrize("M", [1, 2, 40])
@pytest.mark.parametrize("n_layers,fraction", [(8, 0.5), (8, 0.25), (8, 0.125), (5, 0.5)])
def test_mixed_stack_layer_by_layer(gpu, M, n_layers, fraction):
    """A stack of (hidden -> hidden) layers and one gated pair per layer, widths 4 then 2."""
    import torch
    import paper_2601_22716_amd as L
    hidden, inter, r = 288, 200, 24
    bits, avg = L.lords_mixed_schedule(n_layers, fraction)
    assert bits == onp.mixed_schedule(n_layers, fraction) and avg == onp.average_bits(bits)
    say(f"M={M} layers={n_layers} fraction={fraction}: widths {bits}, mean {avg}")
    for l, b in enumerate(bits):
        proj = li.make_case("tiny", M=M, N=hidden, K=hidden, r=r, bits=b, factor_dtype="bf16", seed=900 + l,
                            signed_factors=True)
        gate = li.make_case("tiny", M=M, N=inter, K=hidden, r=r, bits=b, factor_dtype="bf16", seed=1900 + l,
                            signed_factors=True)
        up = li.make_case("tiny", M=M, N=inter, K=hidden, r=r, bits=b, factor_dtype="bf16", seed=2900 + l,
                          signed_factors=True)
        dp, dg, du = gpu.DeviceCase(proj), gpu.DeviceCase(gate), gpu.DeviceCase(up)
        Y = torch.full((M, hidden), float("nan"), dtype=torch.float32, device="cuda")
        L.lords_matmul(dp.X, dp.codes, dp.codebook, dp.B, dp.A, Y, M, hidden, hidden, r, b)
        H = torch.full((M, inter), float("nan"), dtype=torch.float32, device="cuda")
        L.lords_gate_up(dp.X, dg.codes, dg.B, dg.A, du.codes, du.B, du.A, dg.codebook, H, M, inter, hidden, r, b)
        torch.cuda.synchronize()
        check(Y.cpu().numpy(), onp.matmul(proj.X_f32, proj.codes, proj.codebook, proj.B_f32, proj.A_f32, b), f"layer {l} ({b} bits) Y")
        G = onp.matmul(proj.X_f32, gate.codes, gate.codebook, gate.B_f32, gate.A_f32, b)
        U = onp.matmul(proj.X_f32, up.codes, up.codebook, up.B_f32, up.A_f32, b)
        want = onp.silu(G) * U
        got = H.cpu().numpy()
        rms = lambda a: float(np.sqrt(np.mean(np.square(a))))
        bound = Y_MAX_TOL * (1.1 * rms(G) * np.abs(U) + rms(U) * np.abs(onp.silu(G))) * 1.05 + 1e-6
        assert np.isfinite(got).all()
        assert (np.abs(got - want) <= bound).all(), (l, b, float(np.max(np.abs(got - want) / bound)))
        assert onp.rel_fro(got, want) <= 1e-2
