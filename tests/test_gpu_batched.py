"""GPU parity of the shared-input entry points (lords_matmul_batched, lords_gate_up), called
through the C ABI, against the fp64 oracle on the same seeded inputs.

Gates for the products, as for lords_matmul: relative Frobenius error <= 5e-3 and
max |d| <= 2e-2 * rms(oracle).  Where one launch serves all matrices each row is summed in the
same order as in a single-matrix call, so the two must agree to the last bit.

Gates for H = silu(G) * U follow from those of its two products G and U (both computed exactly as
lords_matmul computes them, then combined in fp32): with |dG| <= 2e-2 rms(G), |dU| <= 2e-2 rms(U),
|silu'| <= 1.1 and |silu(g)| <= |g|,
    |dH| <= 1.1 |dG| |U| + |silu(G)| |dU| (+ second order)
         <= 2e-2 * (1.1 rms(G) |U| + rms(U) |silu(G)|) * 1.05 + 1e-6,      element by element,
and the relative Frobenius error is bounded by the sum of the two products' gates, 1e-2.
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


def check(Y, want, what):
    rf, mx = onp.rel_fro(Y, want), onp.max_abs_over_rms(Y, want)
    say(f"   {what}: rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(Y).all(), what
    assert rf <= Y_TOL, (what, rf)
    assert mx <= Y_MAX_TOL, (what, mx)


def layers_sharing_x(Ns, K, r, bits, M, fdt="bf16", seed=0, signed=True):
    """One case per matrix (own codes and factors, drawn from separate seeds); the activations
    are those of the first."""
    cases = [li.make_case("tiny", M=M, N=N, K=K, r=r, bits=bits, factor_dtype=fdt, seed=seed + 17 * i,
                          signed_factors=signed) for i, N in enumerate(Ns)]
    return cases


def run_batched(gpu, cases, M, dtype=None):
    import torch
    import paper_2601_22716_amd as L
    dtype = dtype or torch.float32
    dev = [gpu.DeviceCase(c) for c in cases]
    X = dev[0].X
    Ys = [torch.full((M, d.N), float("nan"), dtype=dtype, device="cuda") for d in dev]
    L.lords_matmul_batched(X, [d.codes for d in dev], dev[0].codebook, [d.B for d in dev], [d.A for d in dev], Ys,
                           [d.N for d in dev], M, dev[0].K, dev[0].r, dev[0].bits)
    torch.cuda.synchronize()
    return dev, [y.float().cpu().numpy() for y in Ys]


BATCHES = [
    # Ns, K, r
    ([300, 70, 70], 544, 32),                       # q/k/v-like proportions, several column blocks
    ([16], 32, 1),                                  # a single matrix goes the ordinary way
    ([100, 200, 50, 77, 33, 64, 130, 90], 2080, 20),  # the most matrices one call takes
    ([200, 120], 1056, 64),                         # rank above 32: four column blocks per workgroup
    ([90, 60, 1], 288, 13),                         # rank not a multiple of 8, a one-row matrix
    ([2000, 40], 4128, 32),                         # very unequal row counts, K not a multiple of a column block
    ([50, 30, 70], 256, 16),                        # one column block: every workgroup writes its rows itself
    ([40, 20], 128, 40),
]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("Ns,K,r", BATCHES)
def test_batched_one_token(gpu, bits, Ns, K, r):
    say(f"batched M=1 bits={bits} Ns={Ns} K={K} r={r}")
    cases = layers_sharing_x(Ns, K, r, bits, 1, seed=3)
    dev, Ys = run_batched(gpu, cases, 1)
    X = cases[0].X_f32
    want = onp.matmul_batched(X, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, bits)
    rms_all = float(np.sqrt(np.mean(np.concatenate([w.ravel() for w in want]) ** 2)))
    for l, (Y, w) in enumerate(zip(Ys, want)):
        if w.size >= 16:
            check(Y, w, f"matrix {l}")
        else:
            # a handful of outputs: a Frobenius ratio over them is one sample of the element-wise
            # error, so only the element-wise gate applies (against the rms of the whole batch)
            mx = float(np.abs(Y - w).max()) / rms_all
            say(f"   matrix {l} ({w.size} outputs): max/rms={mx:.2e}")
            assert mx <= Y_MAX_TOL, (l, mx)
        same_as_single(Y, dev[l].matmul(X=dev[0].X, M=1), 1, f"matrix {l}")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [2, 5, 16])
@pytest.mark.parametrize("Ns,K,r", [([300, 70, 70], 544, 32), ([100, 200, 50, 77, 33, 64, 130, 90], 2080, 20),
                                    ([200, 120], 1056, 64), ([90, 60, 1], 288, 13), ([700, 40], 4128, 24)])
def test_batched_few_tokens(gpu, bits, M, Ns, K, r):
    say(f"batched M={M} bits={bits} Ns={Ns} K={K} r={r}")
    cases = layers_sharing_x(Ns, K, r, bits, M, seed=31)
    dev, Ys = run_batched(gpu, cases, M)
    want = onp.matmul_batched(cases[0].X_f32, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, bits)
    rms_all = float(np.sqrt(np.mean(np.concatenate([w.ravel() for w in want]) ** 2)))
    for l, (Y, w) in enumerate(zip(Ys, want)):
        if w.size >= 16:
            check(Y, w, f"matrix {l}")
        else:
            mx = float(np.abs(Y - w).max()) / rms_all
            assert mx <= Y_MAX_TOL, (l, mx)
        same_as_single(Y, dev[l].matmul(X=dev[0].X, M=M), M, f"matrix {l}")


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("M,fdt,r", [(5, "f32", 24), (1, "f32", 24), (40, "bf16", 24), (20, "bf16", 24), (3, "bf16", 72)])
def test_batched_other_cases_run_matrix_by_matrix(gpu, bits, M, fdt, r):
    say(f"batched M={M} bits={bits} factors={fdt} r={r}")
    cases = layers_sharing_x([150, 64, 33], 544, r, bits, M, fdt=fdt, seed=4)
    _, Ys = run_batched(gpu, cases, M)
    want = onp.matmul_batched(cases[0].X_f32, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, bits)
    for l, (Y, w) in enumerate(zip(Ys, want)):
        check(Y, w, f"matrix {l}")


def test_batched_bf16_output_and_repeatability(gpu):
    import torch
    cases = layers_sharing_x([300, 70, 70], 1056, 32, 4, 1, seed=5)
    _, Y1 = run_batched(gpu, cases, 1, dtype=torch.bfloat16)
    # other calls in between use the same workspace and tickets
    gpu.DeviceCase(cases[0]).matmul()
    _, Y2 = run_batched(gpu, cases, 1, dtype=torch.bfloat16)
    want = onp.matmul_batched(cases[0].X_f32, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, 4)
    for a, b, w in zip(Y1, Y2, want):
        np.testing.assert_array_equal(a, b)
        check(a, w, "bf16 out")


H_TOL = 1e-2


def check_h(H, G, U, what, out_ulp=0.0):
    """H from the GPU against silu(G) * U of the oracle's products G and U (fp64).
    out_ulp: relative rounding step of the output type (2^-8 for bf16), added to the bound."""
    want = onp.silu(G) * U
    rms = lambda a: float(np.sqrt(np.mean(a * a)))
    bound = Y_MAX_TOL * (1.1 * rms(G) * np.abs(U) + rms(U) * np.abs(onp.silu(G))) * 1.05 + 1e-6
    bound = bound + np.abs(want) * out_ulp
    rf = onp.rel_fro(H, want)
    worst = float((np.abs(H - want) / bound).max())
    say(f"   {what}: rel_fro={rf:.2e} worst |dH|/bound={worst:.2f}  (gate rms {rms(G):.2f}, max |g| {np.abs(G).max():.2f})")
    assert np.isfinite(H).all(), what
    assert rf <= H_TOL, (what, rf)
    assert worst <= 1.0, (what, worst)


def oracle_products(cg, cu, bits, rows=None, toks=None):
    X = cg.X_f32 if toks is None else cg.X_f32[toks]
    if rows is None:
        return (onp.matmul(X, cg.codes, cg.codebook, cg.B_f32, cg.A_f32, bits),
                onp.matmul(X, cu.codes, cu.codebook, cu.B_f32, cu.A_f32, bits))
    return (onp.matmul_rows(X, cg.codes, cg.codebook, cg.B_f32, cg.A_f32, bits, rows),
            onp.matmul_rows(X, cu.codes, cu.codebook, cu.B_f32, cu.A_f32, bits, rows))


def run_gate_up(gpu, cg, cu, M, dtype=None):
    import torch
    import paper_2601_22716_amd as L
    dtype = dtype or torch.float32
    dg, du = gpu.DeviceCase(cg), gpu.DeviceCase(cu)
    H = torch.full((M, dg.N), float("nan"), dtype=dtype, device="cuda")
    L.lords_gate_up(dg.X, dg.codes, dg.B, dg.A, du.codes, du.B, du.A, dg.codebook, H, M, dg.N, dg.K, dg.r, dg.bits)
    torch.cuda.synchronize()
    return H.float().cpu().numpy()


def gate_up_cases(N, K, r, bits, M, fdt="bf16", seed=0):
    """Gate and up matrices of one block.  The activations are scaled up (weights are about 0.012
    rms, so a product over K columns is about 0.012 sqrt(K)) so that the gate values spread over
    the curved part of silu, a few units either side of zero, rather than sitting in its linear
    part."""
    cg, cu = layers_sharing_x([N, N], K, r, bits, M, fdt=fdt, seed=seed, signed=False)
    gain = np.float32(250.0 / np.sqrt(K))
    bits16, vals = li.to_bf16(cg.X_f32 * gain)
    cg.X_bf16, cg.X_f32 = bits16, vals
    return cg, cu


GATE_UP = [
    # N, K, r, M
    (200, 544, 32, 1),
    (1000, 256, 8, 1),          # one column block: the pair still meets in the workspace
    (77, 2080, 64, 1),
    (130, 288, 13, 1),
    (150, 544, 24, 6),          # few tokens, one launch
    (300, 2080, 64, 16),
    (90, 288, 13, 2),
    (120, 512, 32, 3),          # one column split: the pair still meets in the workspace
    (150, 544, 24, 20),         # more than one pass of tokens: two products and one element-wise pass
    (96, 320, 32, 40),          # the MFMA GEMM twice
    (48, 64, 4, 1100),          # more tokens than one pass of the workspace takes
    (64, 320, 72, 1),           # a rank the one-launch kernel does not take
]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,r,M", GATE_UP)
def test_gate_up_parity(gpu, bits, N, K, r, M):
    say(f"gate_up bits={bits} N={N} K={K} r={r} M={M}")
    cg, cu = gate_up_cases(N, K, r, bits, M, seed=6)
    H = run_gate_up(gpu, cg, cu, M)
    G, U = oracle_products(cg, cu, bits)
    # the oracle's own gate_up is the reference; its two products give the propagated bound
    want = onp.gate_up(cg.X_f32, (cg.codes, cg.B_f32, cg.A_f32), (cu.codes, cu.B_f32, cu.A_f32), cg.codebook, bits)
    np.testing.assert_allclose(onp.silu(G) * U, want, rtol=1e-12, atol=1e-300)
    check_h(H, G, U, "H")


@pytest.mark.parametrize("fdt", ["bf16", "f32"])
def test_gate_up_bf16_output_and_f32_factors(gpu, fdt):
    import torch
    cg, cu = gate_up_cases(300, 544, 16, 4, 1, fdt=fdt, seed=7)
    H = run_gate_up(gpu, cg, cu, 1, dtype=torch.bfloat16)
    H2 = run_gate_up(gpu, cg, cu, 1, dtype=torch.bfloat16)
    np.testing.assert_array_equal(H, H2)
    G, U = oracle_products(cg, cu, 4)
    check_h(H, G, U, f"bf16 out, {fdt} factors", out_ulp=2.0 ** -8)


# ------------------------------------------------------------------ full-size, sampled
@pytest.mark.parametrize("M", [1, 2, 16])
def test_full_size_qkv_sampled(gpu, M):
    """Llama-3-8B-shaped query/key/value projections (4096, 1024, 1024 rows of 4096 columns, 4 bits,
    rank 32), one launch; 192 sampled rows of each against the oracle."""
    Ns, K, r, bits = [4096, 1024, 1024], 4096, 32, 4
    say(f"full-size q/k/v Ns={Ns} M={M}")
    cases = layers_sharing_x(Ns, K, r, bits, M, seed=8)
    dev, Ys = run_batched(gpu, cases, M)
    rng = np.random.default_rng(80)
    for l, (c, Y) in enumerate(zip(cases, Ys)):
        rows = np.unique(np.concatenate([[0, c.N - 1], rng.integers(0, c.N, 190)]))
        want = onp.matmul_rows(cases[0].X_f32, c.codes, c.codebook, c.B_f32, c.A_f32, bits, rows)
        check(Y[:, rows], want, f"matrix {l}, {rows.size} rows")
        same_as_single(Y, dev[l].matmul(X=dev[0].X, M=M), M, f"matrix {l}")


@pytest.mark.parametrize("M", [1, 2, 16, 2048])
def test_full_size_gate_up_sampled(gpu, M):
    """The headline layer shape as a gate/up pair (14336 x 4096, 4 bits, rank 32): up to 16 tokens in
    one launch, and 2048 tokens; sampled rows against the oracle."""
    N, K, r, bits = 14336, 4096, 32, 4
    say(f"full-size gate/up M={M}")
    cg, cu = gate_up_cases(N, K, r, bits, M, seed=9)
    H = run_gate_up(gpu, cg, cu, M)
    assert np.isfinite(H).all()
    rows = np.unique(np.concatenate([[0, N - 1], np.random.default_rng(90).integers(0, N, 126)]))
    toks = np.unique(np.concatenate([[0, M - 1], np.random.default_rng(91).integers(0, M, 30)]))
    G, U = oracle_products(cg, cu, bits, rows=rows, toks=toks)
    check_h(H[np.ix_(toks, rows)], G, U, f"{toks.size} tokens x {rows.size} rows")


def test_full_size_gate_up_shared_read_back(gpu):
    """A gate/up pair whose partial sums are large enough for the few-token kernel to share a chunk's read-back out
    among the workgroups that meet in it (14336 x 4096, 3 bits, rank 48, 16 tokens: 8 column blocks per matrix, 16
    shares per chunk); sampled rows against the oracle."""
    N, K, r, bits, M = 14336, 4096, 48, 3, 16
    say(f"full-size gate/up rank 48 M={M}")
    cg, cu = gate_up_cases(N, K, r, bits, M, seed=19)
    H = run_gate_up(gpu, cg, cu, M)
    assert np.isfinite(H).all()
    rows = np.unique(np.concatenate([[0, 3, 4, N - 1], np.random.default_rng(92).integers(0, N, 126)]))
    toks = np.arange(M)
    G, U = oracle_products(cg, cu, bits, rows=rows, toks=toks)
    check_h(H[np.ix_(toks, rows)], G, U, f"{toks.size} tokens x {rows.size} rows")
    H2 = run_gate_up(gpu, cg, cu, M)
    np.testing.assert_array_equal(H, H2)


def test_full_size_batched_shared_read_back(gpu):
    """Two matrices of many column blocks sharing X at 16 tokens (4096 x 14336 each, 4 bits, rank 32: 14 column
    blocks, 14 shares per chunk) in one launch: sampled rows against the oracle, and the same as matrix by matrix."""
    Ns, K, r, bits, M = [4096, 4096], 14336, 32, 4, 16
    say(f"full-size batched Ns={Ns} K={K} M={M}")
    cases = layers_sharing_x(Ns, K, r, bits, M, seed=18)
    dev, Ys = run_batched(gpu, cases, M)
    rng = np.random.default_rng(81)
    for l, (c, Y) in enumerate(zip(cases, Ys)):
        rows = np.unique(np.concatenate([[0, c.N - 1], rng.integers(0, c.N, 100)]))
        want = onp.matmul_rows(cases[0].X_f32, c.codes, c.codebook, c.B_f32, c.A_f32, bits, rows)
        check(Y[:, rows], want, f"matrix {l}, {rows.size} rows")
        same_as_single(Y, dev[l].matmul(X=dev[0].X, M=M), M, f"matrix {l}")



def test_workspace_bytes_lent_to_gate_up_stay_clear_of_the_tickets(gpu):
    """The two-product form of lords_gate_up borrows workspace for its fp32 products.  A case whose
    own kernels need no workspace (a single column split) must not be given the front of the buffer,
    where the arrival tickets of the split-K kernels live: a later one-launch call would never finish
    its rows.  (Regression test: it once was.)"""
    cg, cu = gate_up_cases(64, 320, 72, 4, 1, seed=21)          # rank the one-launch kernel does not take
    run_gate_up(gpu, cg, cu, 1)
    cg, cu = gate_up_cases(300, 544, 16, 4, 1, seed=22)         # three column blocks: uses the tickets
    H = run_gate_up(gpu, cg, cu, 1)
    G, U = oracle_products(cg, cu, 4)
    check_h(H, G, U, "after a borrowed workspace")
    cases = layers_sharing_x([300, 70], 544, 32, 4, 1, seed=23)
    _, Ys = run_batched(gpu, cases, 1)
    want = onp.matmul_batched(cases[0].X_f32, [(c.codes, c.B_f32, c.A_f32) for c in cases], cases[0].codebook, 4)
    for Y, w in zip(Ys, want):
        check(Y, w, "batched after a borrowed workspace")
