"""CPU oracle for the LoRDS inference path, in fp64.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the GPU kernels are checked against.  It is plain,
slow and written straight from the definitions; it shares no code with the HIP
path and must never be imported by the product package.  Only tests, the smoke
check and the benchmark's CPU-baseline leg may use it.

What it computes (notation: W_hat is N x K with N out-features and K
in-features; the paper's n x m):

  q[n,k]      = the k-th `bits`-wide code of packed row n          (integer)
  S           = B A            B: N x r, A: r x K      (paper Sec. 3.2, Eq. 3)
  W_hat       = C[q] (.) S     element-wise            (paper Sec. 3.3, the
                 objective || W - (BA) (.) Q ||_F^2, and Fig. 1b: the scale
                 is absorbed into dequantisation; Q_ij is a level of the
                 look-up table, Alg. 1 step 2.1)
  Y           = X W_hat^T      the linear layer the kernel replaces
                 (Sec. 4.4, operator benchmark on q_proj)

Packed row format (the build's storage format, not the paper's): a row is a
little-endian bit string, bit b of the row being bit (b mod 8) of byte
(b div 8); code k occupies bits [bits*k, bits*k + bits).  For 4 bits this is
"low nibble first", for 2 bits four codes per byte from the low end, for
3 bits 32 codes per 12 bytes.

All floating-point inputs are widened to fp64 before any arithmetic; bf16
inputs arrive as fp32 arrays holding bf16-exact values, so widening is exact.

The quantisation side (the inverse of the path; Alg. 1 step 2.1 and the
block-wise scale it starts from):

  quantize    Q_ij = argmin over the levels v of (S_ij v - W_ij)^2, as an index,
              ties going to the lowest index                (Alg. 1, step 2.1)
  block_init  S = ComputeScale(W, block size K/r) written as B A with
              B = the block scales and A = the 0/1 block indicator, which is the
              same S as the SVD factors of Alg. 1 step 1 (rank(S) <= r, Sec. 3.1)
  pack_codes  indices -> packed rows (inverse of unpack_codes)

Layers that share their input (every linear layer of a block is quantised on its
own, Sec. 4.3; Q/K/V and Gate/Up of the module list in Table 7 read one input):

  matmul_batched   Y_l = X W_hat_l^T for each layer l, by the definition above
  gate_up          H = silu(X W_hat_gate^T) (.) (X W_hat_up^T),
                   silu(g) = g / (1 + e^-g): the gated MLP the Gate and Up
                   modules belong to (the model's own activation, not part of
                   the paper's method), written out from its definition

Backward of the layer for fine-tuning the scale factors (Sec. 3.4: B and A are the trainable
parameters, Q stays fixed, the update of the weight is Q (.) (B'A' - BA)).  With
Y = X W_hat^T, W_hat = C[q] (.) (B A) and dY the gradient of a scalar loss with respect to Y,
the chain rule gives

  backward_input    dX = dY W_hat                                   [M, K]
  backward_factors  G  = dY^T X         (gradient w.r.t. W_hat)     [N, K]
                    P  = C[q] (.) G     (gradient w.r.t. S = B A)
                    dB = P A^T   [N, r],        dA = B^T P   [r, K]

Mixed-precision stacks (Sec. 4.2, ultra-low-bit setting): the code width is chosen per layer,

  mixed_schedule     4-bit levels for a leading share of the layers, 2-bit levels for the rest
  average_bits       the bit label of such a stack (3 / 2.5 / 2.25 in Table 3)
  factor_parameters  sum of r (N + K) over matrices at the budget-matched rank (#Float in Table 3)

pinned by the table's own labels and #Float column (tests/test_oracle_mixed_pins.py).

Pins (see tests/test_oracle_pins.py): hand-derived byte vectors for the
unpacker, scalar brute force on tiny inputs, the block-wise special case
(paper Sec. 3.1), identity activations, the rank-1 closed form, the all-ones
table (plain low-rank product), linearity, and the paper's rank table
(Appendix A, Table 7) for `equivalent_rank`.
"""
from __future__ import annotations

import numpy as np


def unpack_codes(codes: np.ndarray, K: int, bits: int) -> np.ndarray:
    """codes: uint8 [N, K*bits/8] -> uint8 [N, K] of level indices."""
    if bits not in (2, 3, 4):
        raise ValueError("bits must be 2, 3 or 4")
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, nbytes = codes.shape
    if nbytes * 8 != K * bits:
        raise ValueError("row length does not match K*bits/8")
    # the row as a little-endian bit string, then `bits` consecutive bits per code
    bitstr = np.unpackbits(codes, axis=1, bitorder="little")       # [N, K*bits]
    fields = bitstr.reshape(N, K, bits).astype(np.uint8)
    q = np.zeros((N, K), dtype=np.uint8)
    for b in range(bits):
        q |= fields[:, :, b] << b
    return q


def scale_matrix(B: np.ndarray, A: np.ndarray) -> np.ndarray:
    """S = B A in fp64 (Eq. 3)."""
    B64 = np.asarray(B, dtype=np.float64)
    A64 = np.asarray(A, dtype=np.float64)
    if B64.shape[1] != A64.shape[0]:
        raise ValueError("rank mismatch between B and A")
    return B64 @ A64


def dequant(codes, codebook, B, A, bits: int) -> np.ndarray:
    """W_hat = C[q] (.) (B A), fp64 [N, K]."""
    K = np.asarray(A).shape[1]
    q = unpack_codes(codes, K, bits)
    C = np.asarray(codebook, dtype=np.float64)
    if C.shape != (1 << bits,):
        raise ValueError("codebook must have 2^bits entries")
    return C[q] * scale_matrix(B, A)


def matmul(X, codes, codebook, B, A, bits: int) -> np.ndarray:
    """Y = X W_hat^T, fp64 [M, N]."""
    W = dequant(codes, codebook, B, A, bits)
    return np.asarray(X, dtype=np.float64) @ W.T


def matmul_rows(X, codes, codebook, B, A, bits: int, rows) -> np.ndarray:
    """Columns `rows` of Y (i.e. Y[:, rows]): the definition restricted to the
    chosen out-features.  Used to check full-size GPU runs on sampled outputs
    without forming all of W_hat."""
    rows = np.asarray(rows, dtype=np.int64)
    return matmul(X, np.asarray(codes)[rows], codebook, np.asarray(B)[rows], A, bits)


def matmul_batched(X, layers, codebook, bits: int):
    """[Y_l] for layers = [(codes_l, B_l, A_l), ...] sharing X and the level table:
    nothing but the single-layer definition, layer by layer."""
    return [matmul(X, codes, codebook, B, A, bits) for (codes, B, A) in layers]


def silu(g) -> np.ndarray:
    """g / (1 + exp(-g)) in fp64, evaluated without overflow for large |g|."""
    g = np.asarray(g, dtype=np.float64)
    e = np.exp(-np.abs(g))                     # in (0, 1]
    return np.where(g >= 0, g / (1.0 + e), g * e / (1.0 + e))


def gate_up(X, gate, up, codebook, bits: int) -> np.ndarray:
    """H = silu(X W_hat_gate^T) (.) (X W_hat_up^T), fp64 [M, N]; gate, up = (codes, B, A)."""
    G = matmul(X, gate[0], codebook, gate[1], gate[2], bits)
    U = matmul(X, up[0], codebook, up[1], up[2], bits)
    return silu(G) * U


def backward_input(dY, codes, codebook, B, A, bits: int) -> np.ndarray:
    """dX = dY W_hat, fp64 [M, K]: gradient of a loss with respect to X given dY = dLoss/dY."""
    W = dequant(codes, codebook, B, A, bits)
    return np.asarray(dY, dtype=np.float64) @ W


def backward_factors(dY, X, codes, codebook, B, A, bits: int):
    """(dB, dA), fp64 [N, r] and [r, K]: gradients with respect to the scale factors (Sec. 3.4)."""
    A64 = np.asarray(A, dtype=np.float64)
    B64 = np.asarray(B, dtype=np.float64)
    K = A64.shape[1]
    q = unpack_codes(codes, K, bits)
    C = np.asarray(codebook, dtype=np.float64)
    G = np.asarray(dY, dtype=np.float64).T @ np.asarray(X, dtype=np.float64)     # dLoss/dW_hat
    P = C[q] * G                                                                  # dLoss/dS
    return P @ A64.T, B64.T @ P


def backward_input_cols(dY, codes, codebook, B, A, bits: int, cols) -> np.ndarray:
    """Columns `cols` of dX (dX[:, cols]): the definition restricted to chosen in-features, for
    checking full-size runs on sampled outputs without forming all of W_hat."""
    cols = np.asarray(cols, dtype=np.int64)
    A64 = np.asarray(A, dtype=np.float64)
    q = unpack_codes(codes, A64.shape[1], bits)[:, cols]
    W = np.asarray(codebook, dtype=np.float64)[q] * (np.asarray(B, dtype=np.float64) @ A64[:, cols])
    return np.asarray(dY, dtype=np.float64) @ W


def backward_factors_rows(dY, X, codes, codebook, B, A, bits: int, rows) -> np.ndarray:
    """Rows `rows` of dB: needs only those rows of G = dY^T X."""
    rows = np.asarray(rows, dtype=np.int64)
    A64 = np.asarray(A, dtype=np.float64)
    q = unpack_codes(np.asarray(codes)[rows], A64.shape[1], bits)
    G = np.asarray(dY, dtype=np.float64)[:, rows].T @ np.asarray(X, dtype=np.float64)
    return (np.asarray(codebook, dtype=np.float64)[q] * G) @ A64.T


def backward_factors_cols(dY, X, codes, codebook, B, A, bits: int, cols) -> np.ndarray:
    """Columns `cols` of dA: needs only those columns of G = dY^T X."""
    cols = np.asarray(cols, dtype=np.int64)
    K = np.asarray(A).shape[1]
    q = unpack_codes(codes, K, bits)[:, cols]
    G = np.asarray(dY, dtype=np.float64).T @ np.asarray(X, dtype=np.float64)[:, cols]
    return np.asarray(B, dtype=np.float64).T @ (np.asarray(codebook, dtype=np.float64)[q] * G)


def equivalent_rank(N: int, K: int, group: int) -> int:
    """Rank whose factor budget r (N + K) matches the block-wise scale budget
    N K / group: r = floor(N K / (group (N + K)))  (Sec. 3.2; Appendix A)."""
    return (int(N) * int(K)) // (int(group) * (int(N) + int(K)))


def mixed_schedule(n_layers: int, fraction_first: float, bits_first: int = 4, bits_rest: int = 2) -> list:
    """Code width of every layer of a mixed-precision stack: the first `fraction_first` of the layers
    (a count rounded half up) use `bits_first`, the remainder `bits_rest` (Sec. 4.2, ultra-low-bit
    setting: 4-bit levels for the first 50 % / 25 % / 12.5 % of the layers and 2-bit levels for the
    rest give the 3 / 2.5 / 2.25-bit rows of Table 3)."""
    n_layers = int(n_layers)
    n_first = int(np.floor(float(fraction_first) * n_layers + 0.5))
    n_first = max(0, min(n_layers, n_first))
    return [int(bits_first)] * n_first + [int(bits_rest)] * (n_layers - n_first)


def average_bits(layer_bits) -> float:
    """Mean code width over layers of equal size (the bit label of a row of Table 3)."""
    layer_bits = list(layer_bits)
    return float(sum(layer_bits)) / float(len(layer_bits))


def factor_parameters(shapes, group: int) -> int:
    """Floating-point parameters of the factors over a list of (N, K) matrices, each at the rank
    that matches a block-wise scale budget of block size `group`: sum of r (N + K)  (Sec. 3.2; the
    #Float column of Table 3 counts these over all linear layers of the model)."""
    return sum(equivalent_rank(N, K, group) * (int(N) + int(K)) for N, K in shapes)


# ----------------------------------------------------------------------------
# error measures used by the parity gates
# ----------------------------------------------------------------------------
def pack_codes(q: np.ndarray, bits: int) -> np.ndarray:
    """uint8 [N, K] of level indices -> packed rows uint8 [N, K*bits/8] (inverse of unpack_codes)."""
    if bits not in (2, 3, 4):
        raise ValueError("bits must be 2, 3 or 4")
    q = np.ascontiguousarray(q, dtype=np.uint8)
    N, K = q.shape
    if (K * bits) % 8:
        raise ValueError("K*bits must be a whole number of bytes")
    if q.size and int(q.max()) >= (1 << bits):
        raise ValueError("index out of range")
    fields = np.zeros((N, K, bits), dtype=np.uint8)
    for b in range(bits):
        fields[:, :, b] = (q >> b) & 1
    return np.packbits(fields.reshape(N, K * bits), axis=1, bitorder="little")


def quantize(W, codebook, B, A, with_margin: bool = False):
    """Alg. 1 step 2.1 in fp64: idx[n,k] = argmin_i (S[n,k] * C[i] - W[n,k])^2, ties to the lowest i.

    with_margin=True also returns, per element, (second smallest error - smallest error), which
    tells a test how close the decision was."""
    S = scale_matrix(B, A)
    W64 = np.asarray(W, dtype=np.float64)
    C = np.asarray(codebook, dtype=np.float64)
    err = (S[:, :, None] * C[None, None, :] - W64[:, :, None]) ** 2         # [N, K, 2^bits]
    idx = np.argmin(err, axis=2).astype(np.uint8)                           # first minimum = lowest index
    if not with_margin:
        return idx
    part = np.partition(err, 1, axis=2)
    return idx, part[:, :, 1] - part[:, :, 0]


def block_scales(W, codebook, group: int) -> np.ndarray:
    """ComputeScale of Alg. 1 step 1, read as symmetric absmax scaling (Sec. 3.1): the scale of a block
    of `group` consecutive columns of a row is max|W_b| / max|level|.  Returns [N, K/group], fp64."""
    W64 = np.asarray(W, dtype=np.float64)
    N, K = W64.shape
    if K % group:
        raise ValueError("K must be a multiple of the block size")
    cmax = float(np.max(np.abs(np.asarray(codebook, dtype=np.float64))))
    return np.abs(W64).reshape(N, K // group, group).max(axis=2) / cmax


def block_init(W, codebook, r: int):
    """S = ComputeScale(W, block size K/r) as factors: B = block scales (N x r), A = block indicator (r x K)."""
    K = np.asarray(W).shape[1]
    if K % r:
        raise ValueError("K must be a multiple of r")
    g = K // r
    B = block_scales(W, codebook, g)
    A = (np.arange(K)[None, :] // g == np.arange(r)[:, None]).astype(np.float64)
    return B, A


def repack_codes(codes: np.ndarray, N: int, K: int, bits: int) -> np.ndarray:
    """The slab-tile layout of the packed codes (a storage format of this build, not the paper's; the
    paper's kernels are only said to be fused, Sec. 4.4): the matrix is cut into slabs of 16 rows and
    column tiles of 128 columns; tile (s, t) is stored whole, tiles in the order s * ceil(K/128) + t; inside
    a tile the 64 chunks of 32 codes (4*bits bytes, as they stand in the canonical row) are ordered
    g * 16 + c for row 16 s + c and 32-code group 4 t + g.  Rows >= N and groups >= K/32 are zero bytes.
    A pure permutation (plus padding): codes, levels and scales are those of the canonical rows."""
    cb = 4 * bits                                          # bytes of a 32-code chunk
    nslabs, nct = -(-N // 16), -(-K // 128)
    out = np.zeros(nslabs * nct * 64 * cb, dtype=np.uint8)
    for n in range(N):
        s, c = divmod(n, 16)
        for grp in range(K // 32):
            t, g = divmod(grp, 4)
            dst = (((s * nct + t) * 64) + g * 16 + c) * cb
            out[dst:dst + cb] = codes[n, grp * cb:(grp + 1) * cb]
    return out


def rel_fro(got, want) -> float:
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    denom = np.linalg.norm(want)
    return float(np.linalg.norm(got - want) / denom) if denom > 0 else float(np.linalg.norm(got))


def max_abs_over_rms(got, want) -> float:
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = np.sqrt(np.mean(want * want))
    err = np.max(np.abs(got - want)) if want.size else 0.0
    return float(err / rms) if rms > 0 else float(err)
