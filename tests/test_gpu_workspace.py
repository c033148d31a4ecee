"""GPU tests of the boundary's workspace handling: lords_matmul_ws (the caller's workspace, no allocation
inside the call), forced kernels (GEMV / SMALLM / MFMA), and HIP graphs that were captured with
different workspace needs and must all stay valid."""
import sys

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp
from oracle import lords_oracle_c as oc

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
    assert rf <= Y_TOL and mx <= Y_MAX_TOL, (what, rf, mx)


def fresh_workspace(nbytes):
    import torch
    import paper_2601_22716_amd as L
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ws[:L.lords_workspace_zero_bytes()].zero_()          # the front must be zero at first use
    ws[L.lords_workspace_zero_bytes():].fill_(0xA5)      # the rest is scratch: its contents must not matter
    return ws


@pytest.mark.parametrize("N,K,r,M,bits", [(1000, 2592, 20, 1, 4), (300, 2080, 64, 1, 2), (130, 4128, 32, 2, 3),
                                          (257, 544, 48, 16, 3), (333, 1056, 40, 5, 4), (300, 4128, 32, 200, 4),
                                          (4096, 4096, 32, 1, 4), (4096, 4096, 32, 40, 4)])
def test_matmul_ws_equals_matmul(gpu, N, K, r, M, bits):
    """The caller-owned workspace changes where the kernels meet, not what they compute: bit-identical
    to lords_matmul, on two calls in a row (the front is left at zero by the first)."""
    import torch
    import paper_2601_22716_amd as L
    say(f"matmul_ws N={N} K={K} r={r} M={M} bits={bits}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=41, signed_factors=True)
    d = gpu.DeviceCase(cs)
    ref = d.matmul()
    need = L.lords_workspace_bytes(M, N, K, r, bits)
    assert need >= L.lords_workspace_zero_bytes()
    ws = fresh_workspace(need)
    for rep in range(2):
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        L.lords_matmul_ws(d.X, d.codes, d.codebook, d.B, d.A, Y, M, N, K, r, bits, ws)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(Y.cpu().numpy(), ref, err_msg=f"call {rep}")
    assert int(ws[:L.lords_workspace_zero_bytes()].max()) == 0, "the front of the workspace was not left at zero"
    # a workspace one byte short is refused
    with pytest.raises(L.LordsError) as e:
        L.lords_matmul_ws(d.X, d.codes, d.codebook, d.B, d.A, Y, M, N, K, r, bits, ws[:need - 256])
    assert e.value.status == 8


@pytest.mark.parametrize("bits,r", [(4, 32), (3, 48), (2, 64)])
@pytest.mark.parametrize("M", [1, 2])
def test_forced_kernels_agree_with_the_oracle(gpu, bits, r, M):
    """GEMV, SMALLM and MFMA forced on the same small layer (ragged N, K over several column blocks)."""
    import paper_2601_22716_amd as L
    N, K = 403, 2592
    say(f"forced kernels bits={bits} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=77, signed_factors=True)
    d = gpu.DeviceCase(cs)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    for name, path in (("gemv", L.LORDS_PATH_GEMV), ("smallm", L.LORDS_PATH_SMALLM), ("mfma", L.LORDS_PATH_MFMA)):
        check(d.matmul(path=path), want, name)


def test_forced_gemv_refuses_what_it_cannot_run(gpu):
    import torch
    import paper_2601_22716_amd as L
    cs = li.make_case("tiny", M=5, N=64, K=256, bits=4, r=8, factor_dtype="bf16", seed=1)
    d = gpu.DeviceCase(cs)
    Y = torch.empty((5, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LordsError) as e:
        L.lords_matmul_ex(d.X, d.codes, d.codebook, d.B, d.A, Y, 5, 64, 256, 8, 4, L.LORDS_PATH_GEMV)
    assert e.value.status == 7


def test_graphs_with_different_workspace_needs_stay_valid(gpu):
    """Two HIP graphs are captured, the second with a larger workspace need than anything before it
    (which makes the library's own workspace grow between the captures); both must replay correctly
    afterwards, alternately, with eager calls in between.  The same with caller-owned workspaces."""
    import torch
    import paper_2601_22716_amd as L
    small = li.make_case("tiny", M=1, N=512, K=2592, bits=4, r=32, factor_dtype="bf16", seed=3)
    big = li.make_case("tiny", M=16, N=28672, K=8192, bits=2, r=64, factor_dtype="bf16", seed=4)     # 32 MB of partial sums
    ds, db = gpu.DeviceCase(small), gpu.DeviceCase(big)
    rows = np.unique(np.random.default_rng(5).integers(0, big.N, 200))
    want_s = onp.matmul(small.X_f32, small.codes, small.codebook, small.B_f32, small.A_f32, small.bits)
    want_b = oc.matmul(big.X_f32, big.codes, big.codebook, big.B_f32, big.A_f32, big.bits, rows=rows)
    Ys = torch.empty((1, small.N), dtype=torch.float32, device="cuda")
    Yb = torch.empty((16, big.N), dtype=torch.float32, device="cuda")
    stream = torch.cuda.Stream()

    def call_small(ws=None):
        if ws is None:
            L.lords_matmul(ds.X, ds.codes, ds.codebook, ds.B, ds.A, Ys, 1, small.N, small.K, small.r, small.bits)
        else:
            L.lords_matmul_ws(ds.X, ds.codes, ds.codebook, ds.B, ds.A, Ys, 1, small.N, small.K, small.r, small.bits, ws)

    def call_big(ws=None):
        if ws is None:
            L.lords_matmul(db.X, db.codes, db.codebook, db.B, db.A, Yb, 16, big.N, big.K, big.r, big.bits)
        else:
            L.lords_matmul_ws(db.X, db.codes, db.codebook, db.B, db.A, Yb, 16, big.N, big.K, big.r, big.bits, ws)

    for own in (True, False):
        ws_s = None if own else fresh_workspace(L.lords_workspace_bytes(1, small.N, small.K, small.r, small.bits))
        ws_b = None if own else fresh_workspace(L.lords_workspace_bytes(16, big.N, big.K, big.r, big.bits))
        with torch.cuda.stream(stream):
            call_small(ws_s)                               # warm-up outside the capture (allocates the library's workspace)
            torch.cuda.synchronize()
            g_small = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_small, stream=stream):
                call_small(ws_s)
            call_big(ws_b)                                 # eager, larger need: the library's workspace grows here
            torch.cuda.synchronize()
            g_big = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_big, stream=stream):
                call_big(ws_b)
            for rep in range(3):
                Ys.fill_(float("nan")); Yb.fill_(float("nan"))
                g_small.replay()
                g_big.replay()
                torch.cuda.synchronize()
                check(Ys.cpu().numpy(), want_s, f"own={own} replay {rep} small")
                check(Yb.cpu().numpy()[:, rows], want_b, f"own={own} replay {rep} big")
                call_small(ws_s)                           # eager work between the replays
                torch.cuda.synchronize()
                check(Ys.cpu().numpy(), want_s, f"own={own} eager {rep} small")
