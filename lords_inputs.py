"""Seeded synthetic inputs for the LoRDS inference path.

This module only *makes inputs*: random packed code bytes, random factors and
activations, the level table, and their bf16 encodings.  It holds none of the
method's arithmetic (no unpacking, no scale product, no dequantisation, no
matmul) so that both the CPU oracle's tests and the GPU path can draw the very
same bits from it without sharing any code of the method itself.

Shapes follow the synthetic Llama-3-shaped layers the benchmark is quoted on
(out-features N, in-features K, tokens M, scale rank r, code width `bits`).

Every array is returned in two forms where bf16 matters:
  * ``*_f32``  float32 values that are exactly representable in bf16
               (what the fp64 oracle widens), and
  * ``*_bf16`` the uint16 bit patterns of the same values (what is copied to
               the GPU).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from statistics import NormalDist

import numpy as np

__all__ = [
    "LayerConfig", "CONFIGS", "nf_codebook", "int_codebook", "to_bf16",
    "bf16_bits_to_f32", "row_bytes", "make_case", "make_blockwise_case", "make_output_grad",
]


# ----------------------------------------------------------------------------
# bf16 encoding (round-to-nearest-even on the fp32 bit pattern)
# ----------------------------------------------------------------------------
def to_bf16(x) -> tuple[np.ndarray, np.ndarray]:
    """Round fp32 values to bf16 (RNE). Returns (uint16 bits, fp32 values)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    bits = rounded.astype(np.uint16)
    return bits, bf16_bits_to_f32(bits)


def bf16_bits_to_f32(bits) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# level tables (inputs of the method: the paper's look-up table of the target
# data type; Algorithm 1 "Require" line)
# ----------------------------------------------------------------------------
def nf_codebook(bits: int) -> np.ndarray:
    """NormalFloat-style table: normal quantiles at the 2^bits evenly spaced
    mid-point probabilities (i + 1/2) / 2^bits, normalised to [-1, 1]."""
    n = 1 << bits
    nd = NormalDist()
    q = [nd.inv_cdf((i + 0.5) / n) for i in range(n)]
    top = q[-1]
    return np.asarray([v / top for v in q], dtype=np.float32)


def int_codebook(bits: int) -> np.ndarray:
    """Signed-integer style table: level i stands for the value i - 2^(bits-1)."""
    n = 1 << bits
    return np.asarray([i - n // 2 for i in range(n)], dtype=np.float32)


def row_bytes(K: int, bits: int) -> int:
    """Bytes of one packed row of K codes."""
    assert (K * bits) % 8 == 0
    return K * bits // 8


# ----------------------------------------------------------------------------
# configurations
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerConfig:
    name: str
    cfg_id: int
    N: int
    K: int
    bits: int
    r: int
    Ms: tuple
    factor_dtype: str = "bf16"      # "bf16" or "f32"
    note: str = ""


CONFIGS = {
    c.name: c for c in [
        LayerConfig("tiny", 1, 512, 256, 4, 4, (4,), "f32",
                    "small case the oracle finishes in well under a second"),
        LayerConfig("qproj_4b", 2, 4096, 4096, 4, 32, (1, 4, 16), "bf16",
                    "Llama-3-8B q_proj shape, decode"),
        LayerConfig("gateup_3b", 3, 14336, 4096, 3, 48, (1, 16), "bf16",
                    "Llama-3-8B MLP gate/up shape at 3 bits"),
        LayerConfig("down_3b", 4, 4096, 14336, 3, 48, (1, 16), "bf16",
                    "Llama-3-8B MLP down shape at 3 bits"),
        LayerConfig("gateup_4b", 5, 14336, 4096, 4, 32, (1, 2048), "bf16",
                    "headline: decode M=1 and prefill M=2048 on the gate/up shape"),
        LayerConfig("down_4b", 6, 4096, 14336, 4, 32, (2048,), "bf16",
                    "prefill on the down shape"),
        LayerConfig("l70b_2b", 7, 28672, 8192, 2, 64, (1, 16, 256, 4096), "bf16",
                    "Llama-3-70B-shaped 2-bit layer, decode to prefill crossover"),
    ]
}


@dataclass
class Case:
    cfg: LayerConfig
    M: int
    codes: np.ndarray          # uint8 [N, K*bits/8], packed rows
    codebook: np.ndarray       # float32 [2^bits]
    B_f32: np.ndarray          # float32 [N, r] (bf16-exact when factor_dtype == bf16)
    A_f32: np.ndarray          # float32 [r, K]
    X_f32: np.ndarray          # float32 [M, K], bf16-exact
    X_bf16: np.ndarray         # uint16 [M, K]
    B_bf16: np.ndarray | None = None
    A_bf16: np.ndarray | None = None
    extra: dict = field(default_factory=dict)

    @property
    def N(self): return self.cfg.N
    @property
    def K(self): return self.cfg.K
    @property
    def r(self): return self.B_f32.shape[1]
    @property
    def bits(self): return self.cfg.bits


def _rng(seed: int, cfg_id: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([seed, cfg_id, stream])


def random_codes(rng, N: int, K: int, bits: int) -> np.ndarray:
    """Uniform random codes, drawn directly as packed bytes.

    With K a multiple of 32 every row is a whole number of bytes (and of
    12-byte groups at 3 bits), so uniformly random bytes ARE uniformly random
    k-bit codes whatever the bit order; no packing step is needed."""
    return rng.integers(0, 256, size=(N, row_bytes(K, bits)), dtype=np.uint8)


def make_case(cfg: LayerConfig | str, M: int | None = None, seed: int = 0,
              signed_factors: bool = False, r: int | None = None,
              factor_dtype: str | None = None, N: int | None = None,
              K: int | None = None, bits: int | None = None,
              codebook: str = "nf") -> Case:
    """Draw one synthetic layer + activations.

    Distributions: X ~ N(0,1) rounded to bf16; codes uniform; factors
    A ~ U(0.5,1.5), B ~ U(0.5,1.5) * 0.02 / r (so S is about 0.02 and
    |w| <= 0.03).  ``signed_factors`` draws A, B ~ N(0,1) (B scaled the same
    way) to exercise cancelling, signed scales as an SVD initialisation gives.
    Shape overrides let tests build ragged variants of a named config."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if any(v is not None for v in (r, factor_dtype, N, K, bits)):
        cfg = LayerConfig(cfg.name + "*", cfg.cfg_id,
                          N if N is not None else cfg.N,
                          K if K is not None else cfg.K,
                          bits if bits is not None else cfg.bits,
                          r if r is not None else cfg.r,
                          cfg.Ms,
                          factor_dtype if factor_dtype is not None else cfg.factor_dtype,
                          cfg.note)
    if M is None:
        M = cfg.Ms[0]
    assert cfg.K % 32 == 0, "K must be a multiple of 32"
    rr = cfg.r
    codes = random_codes(_rng(seed, cfg.cfg_id, 0), cfg.N, cfg.K, cfg.bits)
    g = _rng(seed, cfg.cfg_id, 1)
    if signed_factors:
        Bv = g.standard_normal((cfg.N, rr)).astype(np.float32) * np.float32(0.02 / rr)
        Av = g.standard_normal((rr, cfg.K)).astype(np.float32)
    else:
        Bv = (g.uniform(0.5, 1.5, (cfg.N, rr)) * (0.02 / rr)).astype(np.float32)
        Av = g.uniform(0.5, 1.5, (rr, cfg.K)).astype(np.float32)
    Xv = _rng(seed, cfg.cfg_id, 2).standard_normal((M, cfg.K)).astype(np.float32)
    X_bits, X_f32 = to_bf16(Xv)
    cb = nf_codebook(cfg.bits) if codebook == "nf" else int_codebook(cfg.bits)
    if cfg.factor_dtype == "bf16":
        B_bits, B_f32 = to_bf16(Bv)
        A_bits, A_f32 = to_bf16(Av)
    else:
        B_bits = A_bits = None
        B_f32, A_f32 = Bv, Av
    return Case(cfg, M, codes, cb, B_f32, A_f32, X_f32, X_bits, B_bits, A_bits)


def make_blockwise_case(N: int, K: int, bits: int, group: int, M: int = 1,
                        seed: int = 0, cfg_id: int = 100,
                        factor_dtype: str = "bf16") -> Case:
    """The block-wise special case (paper Sec. 3.1, matrix form): A is the 0/1
    group-indicator matrix (r = K/group rows, A[j,k] = 1 iff k // group == j)
    and B holds one scale per (row, group).  Only the *structure* is built
    here; ``extra['block_scales']`` is the same array as B."""
    assert K % group == 0
    r = K // group
    cfg = LayerConfig(f"blockwise_{N}x{K}_g{group}", cfg_id, N, K, bits, r, (M,),
                      factor_dtype, "block-wise equivalence case")
    codes = random_codes(_rng(seed, cfg_id, 0), N, K, bits)
    g = _rng(seed, cfg_id, 1)
    s = (g.uniform(0.5, 1.5, (N, r)) * 0.02).astype(np.float32)
    A = np.zeros((r, K), dtype=np.float32)
    for j in range(r):
        A[j, j * group:(j + 1) * group] = 1.0
    Xv = _rng(seed, cfg_id, 2).standard_normal((M, K)).astype(np.float32)
    X_bits, X_f32 = to_bf16(Xv)
    if factor_dtype == "bf16":
        B_bits, B_f32 = to_bf16(s)
        A_bits, A_f32 = to_bf16(A)
    else:
        B_bits = A_bits = None
        B_f32, A_f32 = s, A
    return Case(cfg, M, codes, nf_codebook(bits), B_f32, A_f32, X_f32, X_bits,
                B_bits, A_bits, extra={"block_scales": B_f32, "group": group})


def make_output_grad(M: int, N: int, seed: int = 0) -> tuple[np.ndarray, np.ndarray]:
    """A stand-in for dLoss/dY of a layer: M x N values ~ N(0,1) rounded to bf16.
    Returns (uint16 bits, fp32 values)."""
    g = np.random.default_rng([seed, 777, M, N]).standard_normal((M, N)).astype(np.float32)
    return to_bf16(g)
