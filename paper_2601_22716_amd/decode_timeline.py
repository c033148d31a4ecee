"""Phase timeline of the one-token kernel (lords_gemv_kernel.h) from device time stamps.

    python -m paper_2601_22716_amd.build --stamps        # builds liblords_stamps.so (no GPU needed)
    python -m paper_2601_22716_amd.decode_timeline [--config gateup_4b] [--tokens 1] [--launches 40]

Loads liblords_stamps.so (the library built with -DLORDS_GV_STAMPS), runs lords_matmul on synthetic
layers of the named shape (weight sets rotate so that no launch finds its codes in a cache) and prints,
over all workgroups of all launches, when each phase boundary is reached, counted from the first
stamp of the launch.  The stamps are s_memrealtime ticks (100 MHz, 10 ns), kept in registers and
written when a workgroup ends; wave 0 and the last wave of each workgroup report.

Boundaries: 0 kernel entered; 1 flags cleared, rows of B requested, level table built (the four builder
waves only); 2 first slab, activations, A tile and the other slabs of the ring requested, the wave's
rows of B arrived and staged in LDS; 3 A tile arrived, folded with x and laid out as MFMA operands,
rows of B and table of ALL waves seen complete (LDS flags); 4 row stream done (look-ups + MFMAs over
all slabs); 5 barrier behind the stream; 6 sums over ranks and waves, hand-over between column blocks,
Y written.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))

NAMES = ["entered", "B asked, table built", "loads out, B staged", "A folded, flags seen", "stream done", "barrier", "end"]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gateup_4b")
    ap.add_argument("--tokens", type=int, default=1)
    ap.add_argument("--launches", type=int, default=40)
    args = ap.parse_args()

    import torch
    import lords_inputs as li
    lib_path = os.path.join(HERE, "liblords_stamps.so")
    if not os.path.exists(lib_path):
        print("liblords_stamps.so is missing: python -m paper_2601_22716_amd.build --stamps", file=sys.stderr)
        return 2
    lib = ctypes.CDLL(lib_path)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.lords_matmul.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.lords_debug_gemv_stamps.argtypes = [vp, ci, ci, ci, ci, ci, ctypes.POINTER(ci)]

    cfg = li.CONFIGS[args.config]
    M, N, K, r, bits = args.tokens, cfg.N, cfg.K, cfg.r, cfg.bits
    per_set = N * K * bits // 8
    nsets = max(2, -(-(640 << 20) // per_set))
    g = torch.Generator(device="cuda").manual_seed(1)
    sets = []
    for _ in range(nsets):
        codes = torch.randint(0, 256, (N, K * bits // 8), dtype=torch.uint8, device="cuda", generator=g)
        B = (torch.rand((N, r), device="cuda", generator=g) * 0.02 + 0.01).to(torch.bfloat16)
        A = (torch.rand((r, K), device="cuda", generator=g) + 0.5).to(torch.bfloat16)
        sets.append((codes, B, A))
    X = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
    codebook = torch.linspace(-1.0, 1.0, 1 << bits, device="cuda", dtype=torch.float32)
    Y = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    stamps = torch.zeros((2048, 16), dtype=torch.int64, device="cuda")

    def launch(i):
        codes, B, A = sets[i % nsets]
        rc = lib.lords_matmul(X.data_ptr(), codes.data_ptr(), codebook.data_ptr(), B.data_ptr(), A.data_ptr(), Y.data_ptr(),
                              M, N, K, r, bits, 0, 1, None)
        if rc != 0:
            raise RuntimeError(f"lords_matmul returned {rc}")

    for i in range(200):                                   # clocks up, lazily created state
        launch(i)
    torch.cuda.synchronize()
    wgs = ci(0)
    lib.lords_debug_gemv_stamps(stamps.data_ptr(), M, N, K, r, bits, ctypes.byref(wgs))
    if wgs.value < 1 or wgs.value > 2048:
        print("this shape does not run on the one-/two-token kernel", file=sys.stderr)
        return 2
    rows = []
    for i in range(args.launches):
        for _ in range(8):
            launch(i)                                      # (back-to-back launches, as in a decoder; the last one is read)
        torch.cuda.synchronize()
        t = stamps[: wgs.value].cpu().numpy().astype(np.float64)
        t0 = t[:, [0, 8]].min()
        rows.append((t - t0) * 0.01)                       # microseconds from the first stamp of the launch
    lib.lords_debug_gemv_stamps(None, M, N, K, r, bits, None)
    t = np.stack(rows)                                     # [launch][workgroup][16]
    print(f"one-token kernel timeline: {args.config} N={N} K={K} bits={bits} r={r} tokens={M}; {wgs.value} workgroups, "
          f"{args.launches} launches over {nsets} rotating weight sets; microseconds from the first stamp of a launch")
    print(f"{'boundary':<24}{'wave':>6}{'min':>8}{'p10':>8}{'median':>8}{'p90':>8}{'max':>8}")
    for b in range(7):
        for w, off in (("0", 0), ("last", 8)):
            v = t[:, :, off + b].ravel()
            print(f"{b} {NAMES[b]:<22}{w:>6}{v.min():8.2f}{np.percentile(v, 10):8.2f}{np.median(v):8.2f}{np.percentile(v, 90):8.2f}{v.max():8.2f}")
    print("phase durations (median over workgroups and launches, wave 0 / last wave):")
    for b in range(1, 7):
        d0 = np.median(t[:, :, b] - t[:, :, b - 1])
        d1 = np.median(t[:, :, 8 + b] - t[:, :, 8 + b - 1])
        print(f"  {NAMES[b - 1]} -> {NAMES[b]}: {d0:.2f} / {d1:.2f}")
    print(f"last workgroup ends at (median over launches): {np.median(t[:, :, [6, 14]].max(axis=(1, 2))):.2f}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
