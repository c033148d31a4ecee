"""lords_matmul_noalloc (the entry point whose scratch is an array inside the library image) against
lords_matmul, through the C ABI: two calls in a row, the second on a smaller problem; a problem beyond
the built-in limit is refused."""
import sys

import numpy as np
import pytest

import lords_inputs as li

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def test_noalloc_equals_matmul_on_two_calls_in_a_row():
    import torch
    import paper_2601_22716_amd as L
    from tests import gpu_util
    assert torch.cuda.is_available(), "this test needs the MI355X"
    # first a layer whose kernels meet through slots / tickets and fp32 partial sums, then a smaller one
    shapes = [(16, 4096, 4096, 32, 4), (1, 1000, 2592, 20, 4), (2, 130, 4128, 32, 3), (5, 333, 1056, 40, 2), (1, 64, 320, 8, 4)]
    for (M, N, K, r, bits) in shapes:
        say(f"noalloc M={M} N={N} K={K} r={r} bits={bits}")
        cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=19, signed_factors=True)
        d = gpu_util.DeviceCase(cs)
        ref = d.matmul()
        assert L.lords_workspace_bytes(M, N, K, r, bits) <= L.lords_noalloc_limit()
        for rep in range(2):
            Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            L.lords_matmul_noalloc(d.X, d.codes, d.codebook, d.B, d.A, Y, M, N, K, r, bits)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(Y.cpu().numpy(), ref, err_msg=f"M={M} N={N} call {rep}")


def test_noalloc_large_m_uses_what_fits():
    """More than 16 tokens: the large-M kernel would like tile-sized hand-over buffers for every
    workgroup; inside the built-in array it plans with fewer of them or with whole tiles, so the sums
    may be taken in another order than lords_matmul's: same gates as against the oracle."""
    import torch
    import paper_2601_22716_amd as L
    from oracle import lords_oracle as onp
    from tests import gpu_util
    for (M, N, K, r, bits) in [(300, 2100, 4096, 32, 4), (40, 520, 1056, 20, 3)]:
        say(f"noalloc M={M} N={N} K={K} r={r} bits={bits}")
        cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=23, signed_factors=True)
        d = gpu_util.DeviceCase(cs)
        ref = d.matmul()
        for rep in range(2):
            Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            L.lords_matmul_noalloc(d.X, d.codes, d.codebook, d.B, d.A, Y, M, N, K, r, bits)
            torch.cuda.synchronize()
            got = Y.cpu().numpy()
            assert onp.rel_fro(got, ref) <= 1e-5, (M, N, rep)
            assert onp.max_abs_over_rms(got, ref) <= 1e-4, (M, N, rep)


def test_noalloc_refuses_what_does_not_fit():
    import torch
    import paper_2601_22716_amd as L
    from tests import gpu_util
    M, N, K, r, bits = 16, 57344, 8192, 32, 4                 # 29 MB of partial sums: beyond the 24 MiB array
    assert L.lords_workspace_bytes(M, N, K, r, bits) > L.lords_noalloc_limit()
    cs = li.make_case("tiny", M=M, N=64, K=K, bits=bits, r=r, factor_dtype="bf16", seed=2)
    d = gpu_util.DeviceCase(cs)
    # (buffers of the small case: the call must be refused before anything is launched)
    Y = torch.empty((M, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LordsError) as e:
        L.lords_matmul_noalloc(d.X, d.codes, d.codebook, d.B, d.A, Y, M, N, K, r, bits)
    assert e.value.status == 8
