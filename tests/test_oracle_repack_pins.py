"""Pins for the oracle's slab-tile layout of the packed codes (repack_codes): a storage format of this
build (the paper only says its kernels are fused, Sec. 4.4), so the pins are the format's own definition
stated a second time at code granularity, offsets worked by hand, and the properties of a permutation."""
import os

import numpy as np
import pytest

from oracle import lords_oracle as onp


def random_codes(N, K, bits, seed):
    return np.random.default_rng(seed).integers(0, 256, (N, K * bits // 8), dtype=np.uint8)


def code_from_tiled(tiled, n, k, K, bits):
    """Code (n, k) read straight out of the slab-tile buffer, bit by bit (independent of repack_codes)."""
    nct = -(-K // 128)
    s, c = divmod(n, 16)
    t, rem = divmod(k, 128)
    g, j = divmod(rem, 32)
    base = (((s * nct + t) * 64) + g * 16 + c) * (4 * bits)
    bit = bits * j
    v = 0
    for b in range(bits):
        byte = tiled[base + (bit + b) // 8]
        v |= ((int(byte) >> ((bit + b) % 8)) & 1) << b
    return v


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(1, 32), (16, 128), (17, 160), (37, 288), (50, 544)])
def test_every_code_sits_where_the_layout_says(bits, N, K):
    codes = random_codes(N, K, bits, seed=N * 1000 + K + bits)
    tiled = onp.repack_codes(codes, N, K, bits)
    q = onp.unpack_codes(codes, K, bits)
    assert tiled.dtype == np.uint8 and tiled.size == -(-N // 16) * -(-K // 128) * 256 * bits
    rng = np.random.default_rng(7)
    picks = {(0, 0), (N - 1, K - 1), (N - 1, 0), (0, K - 1)} | {(int(rng.integers(N)), int(rng.integers(K))) for _ in range(300)}
    for (n, k) in picks:
        assert code_from_tiled(tiled, n, k, K, bits) == q[n, k], (n, k)


def test_hand_worked_offsets(golden_dir):
    N, K = 37, 288
    rows = []
    with open(os.path.join(golden_dir, "repack_offsets.txt")) as f:
        for line in f:
            t = line.split()
            if t and not t[0].startswith("#"):
                rows.append(tuple(int(x) for x in t))
    assert len(rows) >= 8
    for bits in (2, 3, 4):
        cb = 4 * bits
        # every chunk carries its own name: bytes (n, grp, position) folded into one byte each
        codes = np.zeros((N, K * bits // 8), dtype=np.uint8)
        for n in range(N):
            for grp in range(K // 32):
                codes[n, grp * cb:(grp + 1) * cb] = [(n * 9 + grp * 37 + 11 * i + 1) & 0xFF for i in range(cb)]
        tiled = onp.repack_codes(codes, N, K, bits)
        for (b, n, grp, off) in rows:
            if b == bits:
                np.testing.assert_array_equal(tiled[off:off + cb], codes[n, grp * cb:(grp + 1) * cb], err_msg=str((b, n, grp)))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_permutation_with_zero_padding(bits):
    N, K = 37, 288                                           # 3 slabs (11 rows of padding), 3 column tiles (3 groups of padding)
    codes = random_codes(N, K, bits, seed=3) | 1             # no zero byte in the data: padding is told apart
    tiled = onp.repack_codes(codes, N, K, bits)
    assert int((tiled != 0).sum()) == codes.size             # every data byte exactly once, everything else zero
    assert sorted(tiled[tiled != 0].tolist()) == sorted(codes.ravel().tolist())
    # a matrix that fills its tiles exactly has no padding at all
    full = random_codes(32, 256, bits, seed=4)
    assert onp.repack_codes(full, 32, 256, bits).size == full.size


def test_planted_mistakes_are_caught():
    """The code-granular reading above must reject the likely slips: rows and groups swapped inside a
    tile, tiles ordered column-major."""
    N, K, bits = 37, 288, 4
    codes = random_codes(N, K, bits, seed=9)
    q = onp.unpack_codes(codes, K, bits)
    cb, nct, nslabs = 16, 3, 3

    def build(chunk_index, tile_index):
        out = np.zeros(nslabs * nct * 64 * cb, dtype=np.uint8)
        for n in range(N):
            s, c = divmod(n, 16)
            for grp in range(K // 32):
                t, g = divmod(grp, 4)
                dst = (tile_index(s, t) * 64 + chunk_index(g, c)) * cb
                out[dst:dst + cb] = codes[n, grp * cb:(grp + 1) * cb]
        return out

    good = build(lambda g, c: g * 16 + c, lambda s, t: s * nct + t)
    np.testing.assert_array_equal(good, onp.repack_codes(codes, N, K, bits))
    for bad in (build(lambda g, c: c * 4 + g, lambda s, t: s * nct + t), build(lambda g, c: g * 16 + c, lambda s, t: t * nslabs + s)):
        wrong = sum(code_from_tiled(bad, n, k, K, bits) != q[n, k] for n in range(0, N, 3) for k in range(0, K, 7))
        assert wrong > 0
