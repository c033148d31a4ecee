"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle
on the same seeded inputs.

Gates: unpacked indices bit-exact; W within relative Frobenius error 1e-3;
Y within relative Frobenius error 5e-3 and max |dY| <= 2e-2 * rms(Y_oracle).
"""
import sys

import numpy as np
import pytest

import lords_inputs as li
from oracle import lords_oracle as onp
from oracle import lords_oracle_c as oc

pytestmark = pytest.mark.gpu

W_TOL, Y_TOL, Y_MAX_TOL = 1e-3, 5e-3, 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def check_y(Y, want, what):
    rf, mx = onp.rel_fro(Y, want), onp.max_abs_over_rms(Y, want)
    say(f"   {what}: rel_fro={rf:.2e} max/rms={mx:.2e}")
    assert np.isfinite(Y).all(), what
    assert rf <= Y_TOL, (what, rf)
    assert mx <= Y_MAX_TOL, (what, mx)


# ------------------------------------------------------------------ unpack
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(1, 32), (5, 96), (67, 416), (512, 256)])
def test_unpack_bit_exact(gpu, bits, N, K):
    say(f"unpack bits={bits} N={N} K={K}")
    cs = li.make_case("tiny", N=N, K=K, bits=bits, r=1, seed=11)
    got = gpu.DeviceCase(cs).unpack()
    np.testing.assert_array_equal(got, onp.unpack_codes(cs.codes, K, bits))


# ----------------------------------------------------------------- dequant
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r", [(3, 32, 1), (70, 160, 5), (512, 256, 4), (129, 4128, 48)])
def test_dequant_parity(gpu, bits, fdt, N, K, r):
    say(f"dequant bits={bits} factors={fdt} N={N} K={K} r={r}")
    cs = li.make_case("tiny", N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=5, signed_factors=True)
    W = gpu.DeviceCase(cs).dequant()
    want = onp.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    rf = onp.rel_fro(W, want)
    say(f"   rel_fro={rf:.2e}")
    assert rf <= W_TOL


def test_dequant_bf16_output_is_rounded_oracle(gpu):
    import torch
    cs = li.make_case("tiny", seed=2)
    W = gpu.DeviceCase(cs).dequant(dtype=torch.bfloat16)
    want = onp.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    _, want_bf = li.to_bf16(want.astype(np.float32))
    # exact, or one bf16 ulp where fp32 rounding of the scale moved a tie
    ulp = np.abs(want_bf) * 2.0 ** -7
    assert np.all(np.abs(W - want_bf) <= ulp)
    assert np.mean(W == want_bf) > 0.99


@pytest.mark.parametrize("bits,group", [(4, 32), (2, 64), (3, 32)])
def test_dequant_blockwise_case_is_bit_exact(gpu, bits, group):
    """A = group indicator, B = block scales: one non-zero term per sum, so the
    fp32 GPU result must equal C[q]*s rounded once -- the block-wise dequantiser
    (paper Sec. 3.1) -- to the last bit."""
    say(f"dequant blockwise bits={bits} group={group}")
    cs = li.make_blockwise_case(96, 256, bits, group, seed=4)
    W = gpu.DeviceCase(cs).dequant()
    q = onp.unpack_codes(cs.codes, cs.K, bits)
    s = np.repeat(cs.extra["block_scales"], group, axis=1)
    want = (cs.codebook[q].astype(np.float32) * s.astype(np.float32)).astype(np.float32)
    np.testing.assert_array_equal(W, want)


# ------------------------------------------------------------------ matmul
SHAPES = [
    # N, K, r, M
    (16, 32, 1, 1),
    (70, 160, 5, 3),
    (512, 256, 4, 4),
    (257, 544, 48, 16),
    (130, 1056, 64, 2),
    (300, 288, 33, 7),
    # one-token shapes: ranks on both sides of the 16/32/64 tile edges, several column blocks,
    # a ragged last slab, K not a multiple of a wave's column block
    (200, 512, 8, 1),
    (1000, 2592, 20, 1),
    (130, 4128, 32, 1),
    (77, 288, 33, 1),
    (300, 2080, 64, 1),
    (64, 320, 72, 1),
    # few-token shapes: several column splits, ranks on both sides of 32, a rank that is not a multiple of 8
    (100, 2592, 24, 5),
    (333, 1056, 40, 16),
    (48, 3104, 13, 2),
]


@pytest.mark.parametrize("path", ["decode", "prefill"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("fdt", ["bf16", "f32"])
@pytest.mark.parametrize("N,K,r,M", SHAPES)
def test_matmul_parity_small(gpu, path, bits, fdt, N, K, r, M):
    import paper_2601_22716_amd as L
    say(f"matmul path={path} bits={bits} factors={fdt} N={N} K={K} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype=fdt, seed=9, signed_factors=(r % 2 == 1))
    Y = gpu.DeviceCase(cs).matmul(path=L.LORDS_PATH_DECODE if path == "decode" else L.LORDS_PATH_PREFILL)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check_y(Y, want, "Y")


@pytest.mark.parametrize("N,K,r,M", [(270000, 32, 4, 1), (70000, 64, 8, 3)])
def test_matmul_decode_many_rows(gpu, N, K, r, M):
    """More row chunks than resident workgroups: the decode kernels walk several chunks each."""
    import paper_2601_22716_amd as L
    say(f"matmul decode many rows N={N} K={K} r={r} M={M}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=4, r=r, factor_dtype="bf16", seed=21)
    Y = gpu.DeviceCase(cs).matmul(path=L.LORDS_PATH_DECODE)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    check_y(Y, want, "Y")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [1, 2])
@pytest.mark.parametrize("per", [5, 7, 9, 10, 13, 14, 16, 17])
def test_matmul_one_token_ring_depths(gpu, bits, M, per):
    """K = 256 is one column block, so 256 workgroups share the rows: `per` slabs of 16 rows each.  Up to 8 slabs a
    workgroup holds them all (depths 5 and 7 here), beyond that a ring of 6, 7 or 8 slots is refilled: every depth
    and a ragged last slab."""
    import paper_2601_22716_amd as L
    N = 4096 * per - 5
    say(f"matmul one-token ring: {per} slabs per workgroup, bits={bits} M={M} N={N}")
    cs = li.make_case("tiny", M=M, N=N, K=256, bits=bits, r=32, factor_dtype="bf16", seed=40 + per)
    Y = gpu.DeviceCase(cs).matmul(path=L.LORDS_PATH_DECODE)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check_y(Y, want, "Y")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("r", [40, 48, 56])
@pytest.mark.parametrize("per", [3, 7, 10, 14])
def test_matmul_one_token_three_and_four_rank_tiles(gpu, bits, r, per):
    """Ranks 33..48 take three 16-entry rank tiles per slab at one token (runs of 24 bytes of B per lane), ranks
    49..64 four; with and without a refilled ring, ragged last slab."""
    import paper_2601_22716_amd as L
    N = 4096 * per - 3
    say(f"matmul one-token rank tiles: r={r} bits={bits} {per} slabs per workgroup N={N}")
    cs = li.make_case("tiny", M=1, N=N, K=256, bits=bits, r=r, factor_dtype="bf16", seed=70 + per + r)
    Y = gpu.DeviceCase(cs).matmul(path=L.LORDS_PATH_GEMV)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check_y(Y, want, "Y")


@pytest.mark.parametrize("M", [1, 17, 40, 130, 300])
def test_matmul_parity_ragged_tokens(gpu, M):
    import paper_2601_22716_amd as L
    say(f"matmul ragged M={M}")
    cs = li.make_case("tiny", M=M, N=200, K=512, bits=4, r=32, factor_dtype="bf16", seed=3)
    d = gpu.DeviceCase(cs)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    check_y(d.matmul(path=L.LORDS_PATH_AUTO), want, "auto")
    check_y(d.matmul(path=L.LORDS_PATH_DECODE), want, "decode")
    check_y(d.matmul(path=L.LORDS_PATH_PREFILL), want, "prefill")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,r,M,dt", [
    # few tiles and a long K: the GEMM cuts K into ranges and a second kernel adds them
    (130, 4128, 32, 40, "bf16"),       # bf16 output written by the adding kernel
    (77, 2080, 48, 19, "f32"),         # M*N not a multiple of 4: ragged tail of the adding kernel
    (300, 1056, 64, 130, "bf16"),
    (64, 512, 8, 33, "bf16"),          # exactly four K tiles: one range, no second kernel
])
def test_matmul_prefill_with_k_ranges(gpu, bits, N, K, r, M, dt):
    import torch
    import paper_2601_22716_amd as L
    say(f"prefill K ranges bits={bits} N={N} K={K} r={r} M={M} out={dt}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=61, signed_factors=True)
    d = gpu.DeviceCase(cs)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    Y1 = d.matmul(path=L.LORDS_PATH_PREFILL, dtype=tdt)
    check_y(Y1, want, "Y")
    # the ranges are added in a fixed order: run-to-run identical; other calls in between
    d.matmul(path=L.LORDS_PATH_DECODE, M=min(M, 3), X=d.X[:min(M, 3)].contiguous())
    np.testing.assert_array_equal(d.matmul(path=L.LORDS_PATH_PREFILL, dtype=tdt), Y1)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_matmul_prefill_many_tiles_short_k(gpu, bits):
    """Many output tiles over a short K (6136 rows x 2048 tokens, four K tiles): every tile's prologue and
    epilogue with hardly a loop between them; rows sampled across the row groups of a tile and the ragged end."""
    import paper_2601_22716_amd as L
    N, K, r, M = 6144 - 8, 512, 32, 2048
    say(f"prefill many tiles, short K, bits={bits}")
    cs = li.make_case("tiny", M=M, N=N, K=K, bits=bits, r=r, factor_dtype="bf16", seed=62, signed_factors=True)
    Y = gpu.DeviceCase(cs).matmul(path=L.LORDS_PATH_PREFILL)
    assert np.isfinite(Y).all()
    rows = np.unique(np.concatenate([np.arange(0, 192), np.arange(N - 200, N),
                                     np.random.default_rng(620).integers(0, N, 300)]))
    toks = np.unique(np.concatenate([[0, 127, 128, 255, 256, M - 1], np.random.default_rng(621).integers(0, M, 60)]))
    want = onp.matmul_rows(cs.X_f32[toks], cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits, rows)
    check_y(Y[np.ix_(toks, rows)], want, "Y sample")


def test_matmul_tiny_config(gpu):
    import torch
    cs = li.make_case("tiny")
    d = gpu.DeviceCase(cs)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4)
    check_y(d.matmul(), want, "fp32 Y")
    check_y(d.matmul(dtype=torch.bfloat16), want, "bf16 Y")
    # identity activations: Y = W_hat^T
    X = torch.eye(cs.K, dtype=torch.bfloat16, device="cuda")
    Wt = d.matmul(X=X, M=cs.K)
    check_y(Wt, onp.dequant(cs.codes, cs.codebook, cs.B_f32, cs.A_f32, 4).T, "identity X")


def test_matmul_is_deterministic(gpu):
    cs = li.make_case("qproj_4b", M=4, N=1024)
    d = gpu.DeviceCase(cs)
    y1, y2 = d.matmul(), d.matmul()
    np.testing.assert_array_equal(y1, y2)


@pytest.mark.parametrize("bits,group", [(4, 64), (2, 64)])
def test_matmul_blockwise_case(gpu, bits, group):
    """r = K/group with the indicator A: the block-wise quantised layer."""
    say(f"matmul blockwise bits={bits}")
    cs = li.make_blockwise_case(320, 2048, bits, group, M=3, seed=6)
    assert cs.r == 32
    d = gpu.DeviceCase(cs)
    want = onp.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, bits)
    check_y(d.matmul(), want, "blockwise Y")


# ------------------------------------------------- full-size layers, sampled
FULL = [
    ("qproj_4b", 1), ("qproj_4b", 4), ("qproj_4b", 16),
    ("gateup_3b", 1), ("gateup_3b", 16), ("down_3b", 1), ("down_3b", 16),
    ("gateup_4b", 2), ("down_4b", 1), ("qproj_4b", 2),
    ("gateup_4b", 1), ("gateup_4b", 2048), ("down_4b", 2048),
    ("l70b_2b", 1), ("l70b_2b", 16), ("l70b_2b", 256), ("l70b_2b", 4096),
]


@pytest.mark.parametrize("name,M", FULL)
def test_matmul_full_size_sampled(gpu, name, M):
    """The benchmark's launch configuration at full layer size, checked on sampled
    out-features (all tokens) that the C oracle computes one row at a time."""
    say(f"full-size {name} M={M}")
    cs = li.make_case(name, M=M)
    d = gpu.DeviceCase(cs)
    Y = d.matmul()
    rng = np.random.default_rng(123)
    rows = np.unique(np.concatenate([[0, 1, 15, 16, cs.N - 1], rng.integers(0, cs.N, 250)]))
    Xs = cs.X_f32 if M <= 64 else cs.X_f32
    want = oc.matmul(Xs, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, cs.bits, rows=rows)
    assert np.isfinite(Y).all()
    check_y(Y[:, rows], want, f"{name} M={M} sampled {rows.size} rows")
    # indices of the same layer, bit-exact, on a slab of rows
    if M == cs.cfg.Ms[0]:
        got = d.unpack()
        np.testing.assert_array_equal(got[rows], oc.unpack_codes(cs.codes[rows], cs.K, cs.bits))


@pytest.mark.parametrize("name,M", [("gateup_4b", 1), ("qproj_4b", 4), ("qproj_4b", 64), ("down_4b", 2048), ("gateup_4b", 256)])
def test_matmul_in_a_hip_graph_replays_identically(gpu, name, M):
    """bench.py times the calls as HIP-graph replays: a captured call must give, on every replay, with
    the program's own eager calls and synchronisations in between, exactly what the eager call gives
    (the kernels keep their tickets in a workspace that both kinds of launch share)."""
    import torch
    import paper_2601_22716_amd as L
    cfg = li.CONFIGS[name]
    cs = li.make_case(name, M=M, seed=71)
    d = gpu.DeviceCase(cs)
    args = (d.codes, d.codebook, d.B, d.A)
    Y_eager = torch.zeros((M, cfg.N), dtype=torch.float32, device="cuda")
    L.lords_matmul(d.X, *args, Y_eager, M, cfg.N, cfg.K, cfg.r, cfg.bits)      # also allocates the workspace
    torch.cuda.synchronize()
    Y_graph = torch.zeros_like(Y_eager)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        L.lords_matmul(d.X, *args, Y_graph, M, cfg.N, cfg.K, cfg.r, cfg.bits)  # warm, on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            L.lords_matmul(d.X, *args, Y_graph, M, cfg.N, cfg.K, cfg.r, cfg.bits)
    for rep in range(3):
        Y_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y_graph, Y_eager), f"replay {rep}"
        # eager work of the same kind between the replays
        Y2 = torch.zeros_like(Y_eager)
        L.lords_matmul(d.X, *args, Y2, M, cfg.N, cfg.K, cfg.r, cfg.bits)
        torch.cuda.synchronize()
        assert torch.equal(Y2, Y_eager)


@pytest.mark.parametrize("name,M", [("gateup_4b", 1), ("gateup_4b", 8), ("gateup_4b", 2048), ("l70b_2b", 1), ("down_3b", 64)])
def test_power_of_two_scaling_is_exact_at_full_size(gpu, name, M):
    """A property that needs no oracle and holds for every output of a full-size call: scaling B, A or X
    by a power of two scales every rounding step's input and output alike (no overflow or underflow at
    these magnitudes), so Y must scale exactly, bit for bit."""
    import torch
    import paper_2601_22716_amd as L
    cfg = li.CONFIGS[name]
    cs = li.make_case(name, M=M, seed=72, signed_factors=True)
    d = gpu.DeviceCase(cs)

    def run(X, B, A, codebook=None):
        Y = torch.full((M, cfg.N), float("nan"), dtype=torch.float32, device="cuda")
        L.lords_matmul(X, d.codes, d.codebook if codebook is None else codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)
        torch.cuda.synchronize()
        return Y

    Y0 = run(d.X, d.B, d.A)
    assert torch.isfinite(Y0).all()
    assert torch.equal(run(d.X, d.B * 8, d.A), Y0 * 8), "B scaled by 8"
    assert torch.equal(run(d.X, d.B, d.A * 0.25), Y0 * 0.25), "A scaled by 1/4"
    assert torch.equal(run(d.X * 0.0625, d.B, d.A), Y0 * 0.0625), "X scaled by 1/16"
    # the level table, narrowed to 16 bits inside the kernels (fp16 or bf16): a global scale moved between
    # the table and B changes nothing while the levels stay inside the fp16 range the header asks for
    assert torch.equal(run(d.X, d.B * 2.0 ** -10, d.A, d.codebook * 1024.0), Y0), "levels x 2^10, B x 2^-10"
    assert torch.equal(run(d.X, d.B * 64.0, d.A, d.codebook * 2.0 ** -6), Y0), "levels x 2^-6, B x 2^6"
    # (negating X is NOT such a scaling here: the matrix cores' internal sums are not sign-symmetric to
    #  the last bit, so -X gives -Y only up to rounding)
    Yn = run(-d.X, d.B, d.A)
    assert float((Yn + Y0).abs().max()) <= 1e-5 * float(Y0.abs().max()), "X negated"


def sample_rows(N, count, seed):
    """Row slabs spread over N: the first and last rows, rows on both sides of the 16-row slab and
    256-row tile edges, and random ones."""
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 15, 16, 17, 255, 256, 257, N // 2 - 1, N // 2, N - 257, N - 256, N - 17, N - 16, N - 2, N - 1]
    rows = np.concatenate([[r for r in fixed if 0 <= r < N], rng.integers(0, N, count)])
    return np.unique(rows).astype(np.int64)


@pytest.mark.parametrize("name", ["qproj_4b", "gateup_3b", "down_3b", "gateup_4b", "down_4b", "l70b_2b"])
def test_dequant_full_size_sampled(gpu, name):
    """lords_dequant at the full size of every named layer shape: the whole W finite, and sampled rows
    within the W gate (relative Frobenius error 1e-3) of the fp64 oracle."""
    import torch
    import paper_2601_22716_amd as L
    say(f"full-size dequant {name}")
    cs = li.make_case(name, M=1)
    d = gpu.DeviceCase(cs)
    W = torch.full((cs.N, cs.K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_dequant(d.codes, d.codebook, d.B, d.A, W, cs.N, cs.K, cs.r, cs.bits)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(W).all())
    rows = sample_rows(cs.N, 120, 31)
    got = W[torch.from_numpy(rows).cuda()].cpu().numpy()
    del W
    want = oc.dequant(cs.codes[rows], cs.codebook, cs.B_f32[rows], cs.A_f32, cs.bits)
    rf = onp.rel_fro(got, want)
    say(f"   {rows.size} rows: W rel_fro={rf:.2e}")
    assert rf <= W_TOL, rf


def test_blockwise_equivalence_full_size(gpu):
    """The block-wise special case at the 70B-shaped layer: 28672 x 8192, 2-bit codes, blocks of 64,
    written as factors (A = 0/1 block indicator, rank 128, B = block scales; Sec. 3.1, Alg. 1 step 1
    with block = K/r).  Every scale sum has ONE non-zero term, so the fp32 dequantised weight must be
    C[q] * s rounded once, to the last bit; the product at one token must sit inside the Y gates."""
    import torch
    import paper_2601_22716_amd as L
    N, K, bits, group = 28672, 8192, 2, 64
    say(f"full-size block-wise case {N}x{K} bits={bits} group={group}")
    cs = li.make_blockwise_case(N, K, bits, group, M=1, seed=5)
    assert cs.r == K // group == 128
    d = gpu.DeviceCase(cs)
    rows = sample_rows(N, 100, 57)
    rows_t = torch.from_numpy(rows).cuda()
    W = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    L.lords_dequant(d.codes, d.codebook, d.B, d.A, W, N, K, cs.r, bits)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(W).all())
    got = W[rows_t].cpu().numpy()
    del W
    q = oc.unpack_codes(cs.codes[rows], K, bits)
    s = np.repeat(cs.extra["block_scales"][rows], group, axis=1)
    want = (cs.codebook[q].astype(np.float32) * s.astype(np.float32)).astype(np.float32)
    np.testing.assert_array_equal(got, want)
    # the indices themselves, bit-exact
    idx = torch.full((N, K), 255, dtype=torch.uint8, device="cuda")
    L.lords_unpack(d.codes, idx, N, K, bits)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx[rows_t].cpu().numpy(), q)
    del idx
    # the product, one token and a few
    for M in (1, 16):
        csm = li.make_blockwise_case(N, K, bits, group, M=M, seed=5)
        dm = gpu.DeviceCase(csm)
        Y = dm.matmul()
        assert np.isfinite(Y).all()
        wantY = oc.matmul(csm.X_f32, csm.codes, csm.codebook, csm.B_f32, csm.A_f32, bits, rows=rows)
        check_y(Y[:, rows], wantY, f"block-wise M={M}, {rows.size} rows")
