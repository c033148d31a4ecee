"""Boundary checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and rejects bad arguments in the documented order
before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2601_22716_amd as L
from tests.helpers import read_rank_table

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 4096   # a fake, 16-byte aligned, non-null "device pointer": never dereferenced on the error paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lords.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lords_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree():
    names = declared_functions()
    assert set(names) == set(L.binding.EXPORTS)
    lib = ctypes.CDLL(L.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/lords.h but not exported"


def test_version_and_strings():
    assert L.lords_version() >= 100
    for s in range(0, 9):
        assert L.lords_status_string(s) and L.lords_status_string(s) != L.lords_status_string(99)
    assert "unknown" in L.lords_status_string(99)


def test_row_bytes():
    assert L.lords_row_bytes(4096, 4) == 2048
    assert L.lords_row_bytes(4096, 3) == 1536
    assert L.lords_row_bytes(8192, 2) == 2048
    assert L.lords_row_bytes(32, 3) == 12
    assert L.lords_row_bytes(4096, 5) == 0
    assert L.lords_row_bytes(48, 4) == 0
    assert L.lords_row_bytes(0, 4) == 0


def test_equivalent_rank_matches_table7(golden_dir):
    for _, _, N, K, r128, r256 in read_rank_table(os.path.join(golden_dir, "table7_ranks.txt")):
        assert L.lords_equivalent_rank(N, K, 128) == r128
        assert L.lords_equivalent_rank(N, K, 256) == r256
    assert L.lords_equivalent_rank(4096, 4096, 64) == 32
    assert L.lords_equivalent_rank(0, 4096, 64) == -1
    assert L.lords_equivalent_rank(4096, 4096, 0) == -1


def test_mixed_schedule_matches_oracle_and_table3(golden_dir):
    """Host-side function: compared with the oracle over a grid, and with the paper's bit labels."""
    import ctypes
    from oracle import lords_oracle as onp
    for n in (1, 2, 5, 7, 32, 80):
        for fr in (0.0, 0.1, 0.125, 0.25, 0.29, 0.3, 0.5, 0.77, 1.0, 1.5):
            for b1, b2 in ((4, 2), (3, 2), (4, 3), (2, 4)):
                bits, avg = L.lords_mixed_schedule(n, fr, b1, b2)
                want = onp.mixed_schedule(n, fr, b1, b2)
                assert bits == want, (n, fr, b1, b2)
                assert avg == onp.average_bits(want)
    with open(os.path.join(golden_dir, "table3_mixed_bits.txt")) as f:
        rows = [t.split() for t in f if t.startswith("mix")]
    assert len(rows) == 3
    for _, label, fraction in rows:
        assert L.lords_mixed_schedule(32, float(fraction))[1] == float(label)
    f = L.library().lords_mixed_schedule
    out = (ctypes.c_int * 4)()
    assert f(4, 0.5, 4, 2, None, None) == 1
    assert f(4, 0.5, 5, 2, out, None) == 2
    assert f(4, 0.5, 4, 1, out, None) == 2
    assert f(0, 0.5, 4, 2, out, None) == 3
    assert f(4, -0.1, 4, 2, out, None) == 3
    assert f(4, float("nan"), 4, 2, out, None) == 3
    assert f(4, 0.5, 4, 2, out, None) == 0 and list(out) == [4, 4, 2, 2]     # avg_bits may be NULL


def test_unpack_argument_checks():
    f = L.library().lords_unpack
    assert f(None, P, 4, 64, 4, None) == 1
    assert f(P, None, 4, 64, 4, None) == 1
    assert f(P, P, 4, 64, 5, None) == 2
    assert f(P, P, 4, 64, 1, None) == 2
    assert f(P, P, 0, 64, 4, None) == 3
    assert f(P, P, 4, 48, 4, None) == 3
    assert f(P, P, 4, 0, 4, None) == 3
    assert f(P + 8, P, 4, 64, 4, None) == 4
    assert f(P, P + 1, 4, 64, 4, None) == 4
    # order: NULL before BITS before SHAPE before ALIGN
    assert f(None, P + 1, 0, 48, 7, None) == 1
    assert f(P + 1, P, 0, 48, 7, None) == 2
    assert f(P + 1, P, 0, 48, 4, None) == 3


def test_dequant_argument_checks():
    f = L.library().lords_dequant
    ok = [P, P, P, P, P, 8, 64, 4, 4, 0, 1, None]
    for i in range(5):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[8] = 8
    assert f(*a) == 2
    for i, v in ((5, 0), (6, 40), (7, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[2] = P + 4
    assert f(*a) == 4
    a = list(ok); a[9] = 2
    assert f(*a) == 5
    a = list(ok); a[10] = -1
    assert f(*a) == 5
    a = list(ok); a[0] = None; a[8] = 9; a[6] = 1; a[9] = 7
    assert f(*a) == 1


def test_quantize_argument_checks():
    f = L.library().lords_quantize
    ok = [P, P, P, P, P, 8, 64, 4, 4, 1, 0, None]
    for i in range(5):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[8] = 5
    assert f(*a) == 2
    for i, v in ((5, 0), (6, 48), (7, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[4] = P + 8
    assert f(*a) == 4
    for i in (9, 10):
        a = list(ok); a[i] = 3
        assert f(*a) == 5


def test_block_init_argument_checks():
    f = L.library().lords_block_init
    ok = [P, P, P, P, 8, 64, 4, 4, 1, 0, None]
    for i in range(4):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[7] = 1
    assert f(*a) == 2
    for i, v in ((4, 0), (5, 40), (6, 0), (6, 3)):          # the last: K not a multiple of r
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[2] = P + 2
    assert f(*a) == 4
    a = list(ok); a[8] = 9
    assert f(*a) == 5


def test_matmul_argument_checks():
    f = L.library().lords_matmul
    fx = L.library().lords_matmul_ex
    ok = [P, P, P, P, P, P, 1, 8, 64, 4, 4, 0, 1, None]
    for i in range(6):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[10] = 0
    assert f(*a) == 2
    for i, v in ((6, -1), (7, 0), (8, 16), (8, 100), (9, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[5] = P + 2
    assert f(*a) == 4
    a = list(ok); a[11] = 3
    assert f(*a) == 5
    a = list(ok); a[12] = 3
    assert f(*a) == 5
    assert fx(*ok, 9) == 5 and fx(*ok, -1) == 5
    # M == 0 is a no-op that succeeds without touching the device
    a = list(ok); a[6] = 0
    assert f(*a) == 0
    # a rank beyond what the kernels hold in registers is reported, not launched
    a = list(ok); a[9] = 100000
    assert f(*a) == 7


def test_workspace_queries_and_matmul_ws_argument_checks():
    """Host-side only: the size queries, and the order NULL -> BITS -> SHAPE -> ALIGN -> DTYPE -> (M == 0) ->
    UNSUPPORTED -> WORKSPACE of the entry points that take their scratch from the caller or from the
    library image.  No argument below lets a launch happen."""
    lib = L.library()
    zero = L.lords_workspace_zero_bytes()
    assert zero > 0 and zero % 256 == 0
    assert L.lords_noalloc_limit() == 24 << 20
    # every problem needs at least the zero front; invalid arguments give 0
    assert L.lords_workspace_bytes(1, 14336, 4096, 32, 4) >= zero
    assert L.lords_workspace_bytes(0, 14336, 4096, 32, 4) == zero
    for bad in ((1, 14336, 4096, 32, 5), (1, 0, 4096, 32, 4), (1, 8, 48, 4, 4), (1, 8, 64, 0, 4), (-1, 8, 64, 4, 4),
                (1, 8, 64, 100000, 4)):
        assert L.lords_workspace_bytes(*bad) == 0, bad
    assert L.lords_workspace_bytes(1, 8, 64, 4, 4, 7) == 0 and L.lords_workspace_bytes(1, 8, 64, 4, 4, 0, 9) == 0
    # the few-token kernels keep partial sums: more than the front; more tokens, more bytes
    w4, w16 = (L.lords_workspace_bytes(m, 14336, 4096, 32, 4) for m in (4, 16))
    assert zero < w4 < w16
    # forcing a kernel changes the need: the one-token kernel needs the front only
    assert L.lords_workspace_bytes(1, 14336, 4096, 32, 4, 0, L.LORDS_PATH_GEMV) == zero
    assert L.lords_workspace_bytes(1, 14336, 4096, 32, 4, 0, L.LORDS_PATH_SMALLM) > zero
    # every shape of the named layers that the few-token kernels take fits the built-in array (the large-M
    # kernel, which also takes a few tokens at ranks above 32 on large layers, plans with what it is given)
    for (m, n, k, r, b) in ((1, 14336, 4096, 32, 4), (16, 14336, 4096, 32, 4), (8, 4096, 14336, 48, 3), (1, 28672, 8192, 64, 2),
                            (16, 4096, 4096, 32, 4)):
        assert 0 < L.lords_workspace_bytes(m, n, k, r, b) <= L.lords_noalloc_limit(), (m, n, k, r, b)

    f = lib.lords_matmul_ws
    W = 256 * 1024          # an aligned fake workspace address; never dereferenced
    ok = [P, P, P, P, P, P, 1, 8, 64, 4, 4, 0, 1, None, 0, W, 1 << 30]
    for i in range(6):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[10] = 0
    assert f(*a) == 2
    for i, v in ((6, -1), (7, 0), (8, 16), (9, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[5] = P + 2
    assert f(*a) == 4
    a = list(ok); a[15] = W + 16
    assert f(*a) == 4
    a = list(ok); a[11] = 3
    assert f(*a) == 5
    a = list(ok); a[14] = 9
    assert f(*a) == 5
    a = list(ok); a[6] = 0
    assert f(*a) == 0
    a = list(ok); a[9] = 100000
    assert f(*a) == 7
    # forced one-token kernel on a shape it does not take (fp32 factors; five tokens)
    a = list(ok); a[11] = 1; a[14] = L.LORDS_PATH_GEMV
    assert f(*a) == 7
    a = list(ok); a[6] = 5; a[14] = L.LORDS_PATH_GEMV
    assert f(*a) == 7
    # a missing or short workspace is refused before anything is launched
    a = list(ok); a[15] = None
    assert f(*a) == 8
    a = list(ok); a[16] = L.lords_workspace_zero_bytes() - 1
    assert f(*a) == 8
    # the entry point without allocation: same checks (no launch: NULL pointers / bad arguments only)
    g = lib.lords_matmul_noalloc
    okg = [P, P, P, P, P, P, 1, 8, 64, 4, 4, 0, 1, None]
    a = list(okg); a[0] = None
    assert g(*a) in (1, 6)              # (6: no GPU here, the array's address cannot be asked for)


def ptr_array(vals):
    arr = (ctypes.c_void_p * len(vals))()
    for i, v in enumerate(vals):
        arr[i] = v
    return arr


def test_repack_queries_and_argument_checks():
    """Host-side only: the size of the slab-tile buffer and the argument order of lords_repack and
    lords_matmul_repacked (NULL -> BITS -> SHAPE -> ALIGN -> DTYPE -> (M == 0) -> UNSUPPORTED); no launch."""
    from oracle import lords_oracle as onp
    import numpy as np
    for (n, k, b) in ((1, 32, 4), (16, 128, 2), (17, 160, 3), (37, 288, 4), (14336, 4096, 4), (28672, 8192, 2)):
        assert L.lords_repack_bytes(n, k, b) == -(-n // 16) * -(-k // 128) * 256 * b
    assert L.lords_repack_bytes(37, 288, 3) == onp.repack_codes(np.zeros((37, 288 * 3 // 8), dtype=np.uint8), 37, 288, 3).size
    for bad in ((0, 64, 4), (4, 48, 4), (4, 64, 5)):
        assert L.lords_repack_bytes(*bad) == 0
    f = L.library().lords_repack
    assert f(None, P, 4, 64, 4, None) == 1 and f(P, None, 4, 64, 4, None) == 1
    assert f(P, P, 4, 64, 7, None) == 2
    assert f(P, P, 0, 64, 4, None) == 3 and f(P, P, 4, 40, 4, None) == 3
    assert f(P + 4, P, 4, 64, 4, None) == 4 and f(P, P + 2, 4, 64, 4, None) == 4
    assert f(None, P + 1, 0, 48, 7, None) == 1 and f(P + 1, P, 0, 48, 7, None) == 2 and f(P + 1, P, 0, 48, 4, None) == 3
    g = L.library().lords_matmul_repacked
    ok = [P, P, P, P, P, P, 1, 8, 64, 4, 4, 0, 1, None, 0]
    for i in range(6):
        a = list(ok); a[i] = None
        assert g(*a) == 1
    a = list(ok); a[10] = 0
    assert g(*a) == 2
    for i, v in ((6, -1), (7, 0), (8, 16), (9, 0)):
        a = list(ok); a[i] = v
        assert g(*a) == 3
    a = list(ok); a[1] = P + 2
    assert g(*a) == 4
    a = list(ok); a[11] = 3
    assert g(*a) == 5
    a = list(ok); a[14] = 9
    assert g(*a) == 5
    a = list(ok); a[6] = 0
    assert g(*a) == 0                                        # M == 0: nothing to do
    a = list(ok); a[11] = 1                                  # fp32 factors belong to kernels that read canonical rows only
    assert g(*a) == 7
    a = list(ok); a[9] = 200                                 # so do ranks above 128
    assert g(*a) == 7


def test_matmul_batched_argument_checks():
    f = L.library().lords_matmul_batched
    three = lambda: ptr_array([P, P, P])
    ns = (ctypes.c_int * 3)(8, 16, 4)

    def ok():
        #       X  codes    cb  B        A        Y        N   L  M  K   r  bits fdt ydt stream
        return [P, three(), P, three(), three(), three(), ns, 3, 1, 64, 4, 4, 0, 1, None]
    for i in (0, 1, 2, 3, 4, 5, 6):
        a = ok(); a[i] = None
        assert f(*a) == 1
    for i in (1, 3, 4, 5):                    # a NULL entry inside an array
        a = ok(); a[i] = ptr_array([P, None, P])
        assert f(*a) == 1
    for L_ in (0, 9, -1):                     # the count is checked before the arrays are read
        a = ok(); a[7] = L_
        assert f(*a) == 3
    a = ok(); a[11] = 5
    assert f(*a) == 2
    for i, v in ((8, -1), (9, 48), (9, 0), (10, 0)):
        a = ok(); a[i] = v
        assert f(*a) == 3
    a = ok(); a[6] = (ctypes.c_int * 3)(8, 0, 4)
    assert f(*a) == 3
    a = ok(); a[3] = ptr_array([P, P + 4, P])
    assert f(*a) == 4
    a = ok(); a[0] = P + 8
    assert f(*a) == 4
    for i in (12, 13):
        a = ok(); a[i] = 7
        assert f(*a) == 5
    a = ok(); a[8] = 0                         # no tokens: nothing to do
    assert f(*a) == 0


def test_gate_up_argument_checks():
    f = L.library().lords_gate_up
    #     X  cg Bg Ag cu Bu Au cb H  M  N  K   r  bits fdt hdt stream
    ok = [P, P, P, P, P, P, P, P, P, 1, 8, 64, 4, 4, 0, 1, None]
    for i in range(9):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[13] = 1
    assert f(*a) == 2
    for i, v in ((9, -1), (10, 0), (11, 16), (12, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    for i in range(9):
        a = list(ok); a[i] = P + 8
        assert f(*a) == 4
    for i in (14, 15):
        a = list(ok); a[i] = 2
        assert f(*a) == 5
    a = list(ok); a[9] = 0
    assert f(*a) == 0


def test_transpose_codes_argument_checks():
    f = L.library().lords_transpose_codes
    ok = [P, P, 64, 64, 4, None]
    for i in (0, 1):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[4] = 8
    assert f(*a) == 2
    for i, v in ((2, 0), (2, 40), (3, 16), (3, 48)):        # N must be a multiple of 32, K too
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[1] = P + 4
    assert f(*a) == 4


def test_backward_input_argument_checks():
    f = L.library().lords_backward_input
    #     dY codes_t cb B  A  dX M  N   K   r  bits fdt xdt stream
    ok = [P, P,      P, P, P, P, 2, 64, 64, 4, 4,   0,  1,  None]
    for i in range(6):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[10] = 0
    assert f(*a) == 2
    for i, v in ((6, -1), (7, 48), (7, 0), (8, 40), (9, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[5] = P + 8
    assert f(*a) == 4
    for i in (11, 12):
        a = list(ok); a[i] = 4
        assert f(*a) == 5
    a = list(ok); a[6] = 0
    assert f(*a) == 0


def test_backward_factors_argument_checks():
    f = L.library().lords_backward_factors
    #     dY X  codes cb B  A  dB dA M  N   K   r  bits fdt stream
    ok = [P, P, P,    P, P, P, P, P, 2, 64, 64, 4, 4,   0,  None]
    for i in range(8):
        a = list(ok); a[i] = None
        assert f(*a) == 1
    a = list(ok); a[12] = 5
    assert f(*a) == 2
    for i, v in ((8, -1), (9, 0), (10, 16), (11, 0)):
        a = list(ok); a[i] = v
        assert f(*a) == 3
    a = list(ok); a[6] = P + 4
    assert f(*a) == 4
    a = list(ok); a[13] = 2
    assert f(*a) == 5
    for i, v in ((9, 36), (11, 65)):                         # rows not a multiple of 8; rank above 64
        a = list(ok); a[i] = v
        assert f(*a) == 7


def test_binding_raises_with_status_name():
    with pytest.raises(L.LordsError) as e:
        L.binding._check(4, "lords_matmul")
    assert "LORDS_ERR_ALIGN" in str(e.value)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py must say so and exit before touching any device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""
