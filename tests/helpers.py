"""Test-side helpers written independently of both the oracle and the HIP path."""
from __future__ import annotations

import numpy as np


def pack_codes_py(q, bits: int) -> np.ndarray:
    """Pure-Python packer: row of codes -> bytes, by setting single bits of a
    big integer (code k goes to bits [bits*k, bits*k+bits) of the row)."""
    q = np.asarray(q)
    N, K = q.shape
    assert (K * bits) % 8 == 0
    out = np.zeros((N, K * bits // 8), dtype=np.uint8)
    for n in range(N):
        big = 0
        for k in range(K):
            v = int(q[n, k])
            assert 0 <= v < (1 << bits)
            big |= v << (bits * k)
        out[n] = np.frombuffer(big.to_bytes(K * bits // 8, "little"), dtype=np.uint8)
    return out


def read_packed_golden(path):
    cases = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, byts, codes = [p.strip() for p in line.split("|")]
            cases.append((int(bits),
                          np.array([int(b, 16) for b in byts.split()], dtype=np.uint8),
                          np.array([int(c) for c in codes.split()], dtype=np.uint8)))
    return cases


def read_rank_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            rows.append((p[0], p[1], int(p[2]), int(p[3]), int(p[4]), int(p[5])))
    return rows
