#!/usr/bin/env python3
"""Benchmark of the LoRDS fused dequantise-and-multiply on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload decode|prefill|all]

A "step" is one lords_matmul call (the whole hot path: unpack, look-up, scale
regeneration, dequantise, multiply) on one synthetic Llama-3-8B gate/up layer
(N = 14336, K = 4096, 4-bit codes, rank 32), M = 1 token: the decode headline.
Consecutive steps walk through enough distinct weight sets (> 600 MB in total)
that no step finds its weights in the 256 MB last-level cache.  Inputs are
resident in HBM before the timed region.  The K timed steps are timed twice,
launched one by one and as one HIP-graph replay; the faster of the two is the
reported number (both are listed), so it is the GPU's, not the interpreter's.

Prints ONE JSON line.  `value` is decode GB/s (algorithmic bytes / time);
`prefill` carries TFLOP/s at M = 2048 on the same layer; `roofline` belongs to
the decode kernel, `prefill.roofline` to the MFMA GEMM; `cpu_baseline` is the
fp64 C oracle timed on this host's cores (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, vendor figure
COLD_BYTES = 600e6             # rotate through at least this many weight bytes

TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "bench_decode_m1_prefill_m2048_gateup4b_hbm_traffic.md")


def counter_traffic():
    """HBM bytes per launch of the two headline kernels, from the tracked rocprofv3 --pmc summary (FETCH_SIZE
    and WRITE_SIZE per dispatch, each scaled by what the same counter reads for a plain copy kernel of known
    size; the file says how).  The summary carries one machine-readable line
        traffic_bytes_per_launch decode=<int> prefill=<int> taken_at=<commit>
    Returns ({"decode": bytes or None, "prefill": bytes or None}, commit or None)."""
    out, commit = {"decode": None, "prefill": None}, None
    try:
        with open(TRAFFIC_SUMMARY) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    for tok in line.split()[1:]:
                        k, _, v = tok.partition("=")
                        if k in out:
                            out[k] = int(v)
                        elif k == "taken_at":
                            commit = v
    except OSError:
        pass
    return out, commit


def algorithmic_bytes(M, N, K, r, bits, factor_bytes=2, y_bytes=4):
    return N * K * bits // 8 + (N * r + r * K) * factor_bytes + M * K * 2 + M * N * y_bytes + (1 << bits) * 4


def make_sets(cfg_name, M, nsets, li, torch):
    """nsets independent weight sets of one layer shape + one activation matrix."""
    import paper_2601_22716_amd as L
    bf16_tensor = L.bf16_from_bits
    sets = []
    cs0 = None
    for s in range(nsets):
        cs = li.make_case(cfg_name, M=M, seed=1000 + s)
        if cs0 is None:
            cs0 = cs
        sets.append((torch.from_numpy(cs.codes).cuda(), bf16_tensor(cs.B_bf16), bf16_tensor(cs.A_bf16)))
    X = bf16_tensor(cs0.X_bf16)
    codebook = torch.from_numpy(cs0.codebook.copy()).cuda()
    return cs0, sets, X, codebook


# The GPU raises its clocks over the first tens of milliseconds of continuous load (the headline
# GEMM takes 283 us per launch right after idle and 217 us from about 60 ms on), so every timed
# region follows untimed repetitions of the same work for this long.
SETTLE_MS = 150.0


def time_region(run, steps, stream, torch):
    """Wall seconds and HIP-event milliseconds of run() (which enqueues `steps` steps on `stream`)."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        t_end = time.perf_counter() + SETTLE_MS * 1e-3
        while time.perf_counter() < t_end:
            run()
            torch.cuda.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        run()
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    return wall, ev0.elapsed_time(ev1)


def time_steps(run_step, steps, warmup, torch, use_graph=True):
    """Times EXACTLY `steps` steps twice: launched one by one from this process, and as one HIP graph
    replay.  Returns (wall seconds, event milliseconds, mode) of the faster of the two, plus both
    per-step wall times.  Either way the region is bracketed by synchronize() on both sides."""
    for i in range(warmup):
        run_step(i)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()

    def eager():
        for i in range(steps):
            run_step(i)
    with torch.cuda.stream(stream):
        eager()                                     # untimed: lazily created state, caches
    best = time_region(eager, steps, stream, torch) + ("eager",)
    per_step = {"eager": best[0] / steps}
    if use_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                eager()
            graph.replay()                          # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        g = time_region(graph.replay, steps, stream, torch) + ("hip_graph",)
        per_step["hip_graph"] = g[0] / steps
        if g[0] < best[0]:
            best = g
    return best[0], best[1], best[2], per_step


def bench_decode(args, L, li, torch):
    name, M = "gateup_4b", 1
    cfg = li.CONFIGS[name]
    per_set = cfg.N * cfg.K * cfg.bits // 8
    nsets = int(-(-COLD_BYTES // per_set))
    cs, sets, X, codebook = make_sets(name, M, nsets, li, torch)
    Y = torch.zeros((M, cfg.N), dtype=torch.float32, device="cuda")

    def run_step(i):
        codes, B, A = sets[i % nsets]
        L.lords_matmul(X, codes, codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)

    wall, ev_ms, mode, per_step = time_steps(run_step, args.steps, args.warmup, torch, use_graph=not args.no_graph)
    ab = algorithmic_bytes(M, cfg.N, cfg.K, cfg.r, cfg.bits)
    sec_per_step = wall / args.steps
    ev_per_launch = ev_ms * 1e-3 / args.steps
    achieved = ab / ev_per_launch / 1e9
    out = {
        "value": ab / sec_per_step / 1e9,
        "ms_per_step": sec_per_step * 1e3,
        "ms_per_step_by_launch_mode": {k: v * 1e3 for k, v in per_step.items()},
        "config": {"workload": f"decode M={M}, Llama-3-8B gate/up shape N={cfg.N} K={cfg.K}, {cfg.bits}-bit codes, rank {cfg.r}, "
                               f"bf16 factors, fp32 Y; {nsets} rotating weight sets (cold last-level cache)",
                   "algorithmic_bytes_per_step": ab, "weight_sets": nsets, "launch_mode": mode},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": counter_traffic()[0]["decode"],
                     "traffic_taken_at": counter_traffic()[1],
                     "kernel": "lords::gemv_kernel<4,2,1,1,1,7,true,true,false,false> (bits, tiles, G, LG, tokens, ring, refill, 16-byte B loads, several matrices, quadruple table)",
                     "us_per_launch": ev_per_launch * 1e6},
    }
    return out, cs, sets[0], X, codebook


def bench_prefill(args, L, li, torch):
    name, M = "gateup_4b", 2048
    cfg = li.CONFIGS[name]
    cs, sets, X, codebook = make_sets(name, M, 2, li, torch)
    Y = torch.zeros((M, cfg.N), dtype=torch.bfloat16, device="cuda")

    def run_step(i):
        codes, B, A = sets[i % 2]
        L.lords_matmul(X, codes, codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)

    steps = max(1, min(args.steps, 20))
    wall, ev_ms, mode, per_step = time_steps(run_step, steps, min(args.warmup, 3), torch, use_graph=not args.no_graph)
    flops = 2.0 * M * cfg.N * cfg.K
    ev_per_launch = ev_ms * 1e-3 / steps
    achieved = flops / ev_per_launch / 1e12
    return {
        "metric": "prefill TFLOP/s (2MNK / time)", "value": flops / (wall / steps) / 1e12, "unit": "TFLOP/s",
        "steps": steps, "ms_per_step": wall / steps * 1e3, "dtype": "bf16",
        "config": {"workload": f"prefill M={M}, N={cfg.N} K={cfg.K}, {cfg.bits}-bit codes, rank {cfg.r}, bf16 Y",
                   "launch_mode": mode},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": counter_traffic()[0]["prefill"],
                     "traffic_taken_at": counter_traffic()[1],
                     "kernel": "lords::prefill_kernel<4,1,1,2,8,16>", "us_per_launch": ev_per_launch * 1e6},
    }


def bench_other(args, L, li, torch):
    """Context figures on the same layer: the other token counts the method is quoted at (not the headline)."""
    name = "gateup_4b"
    cfg = li.CONFIGS[name]
    out = []
    for M in (4, 16, 256, 4096):
        decode = M <= 32
        nsets = int(-(-COLD_BYTES // (cfg.N * cfg.K * cfg.bits // 8))) if decode else 2
        cs, sets, X, codebook = make_sets(name, M, nsets, li, torch)
        Y = torch.zeros((M, cfg.N), dtype=torch.float32 if decode else torch.bfloat16, device="cuda")

        def run_step(i):
            codes, B, A = sets[i % nsets]
            L.lords_matmul(X, codes, codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)

        steps = 100 if decode else 10
        wall, ev_ms, mode, _ = time_steps(run_step, steps, 5, torch, use_graph=not args.no_graph)
        us = ev_ms * 1e3 / steps
        if decode:
            ab = algorithmic_bytes(M, cfg.N, cfg.K, cfg.r, cfg.bits)
            out.append({"workload": f"decode M={M}", "us_per_launch": us, "value": ab / us / 1e3, "unit": "GB/s",
                        "frac_of_hbm_peak": ab / us / 1e3 / HBM_PEAK_GBS})
        else:
            fl = 2.0 * M * cfg.N * cfg.K
            out.append({"workload": f"prefill M={M}", "us_per_launch": us, "value": fl / us / 1e6, "unit": "TFLOP/s",
                        "frac_of_mfma_peak": fl / us / 1e6 / MFMA_BF16_PEAK_TFLOPS})
        del sets, X, Y
    out.extend(bench_repacked(args, L, li, torch))
    out.extend(bench_shared_input(args, L, li, torch))
    out.extend(bench_block(args, L, li, torch))
    out.extend(bench_backward(args, L, li, torch))
    return out


def bench_repacked(args, L, li, torch):
    """The headline layer with its codes in the slab-tile layout (lords_repack, done once, offline):
    the same product from a matrix whose wave-level loads are contiguous."""
    name = "gateup_4b"
    cfg = li.CONFIGS[name]
    out = []
    for M, steps in ((1, 400), (16, 100), (2048, 20)):
        decode = M <= 32
        nsets = int(-(-COLD_BYTES // (cfg.N * cfg.K * cfg.bits // 8))) if decode else 2
        cs, sets, X, codebook = make_sets(name, M, nsets, li, torch)
        tiled = []
        for codes, B, A in sets:
            t = torch.empty(L.lords_repack_bytes(cfg.N, cfg.K, cfg.bits), dtype=torch.uint8, device="cuda")
            L.lords_repack(codes, t, cfg.N, cfg.K, cfg.bits)
            tiled.append((t, B, A))
        torch.cuda.synchronize()
        del sets
        Y = torch.zeros((M, cfg.N), dtype=torch.float32 if decode else torch.bfloat16, device="cuda")

        def run_step(i):
            t, B, A = tiled[i % nsets]
            L.lords_matmul_repacked(X, t, codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits)

        wall, ev_ms, mode, _ = time_steps(run_step, steps, 5, torch, use_graph=not args.no_graph)
        us = ev_ms * 1e3 / steps
        if decode:
            ab = algorithmic_bytes(M, cfg.N, cfg.K, cfg.r, cfg.bits)
            out.append({"workload": f"decode M={M}, codes in the slab-tile layout (lords_repack)", "us_per_launch": us, "launch_mode": mode,
                        "value": ab / us / 1e3, "unit": "GB/s", "frac_of_hbm_peak": ab / us / 1e3 / HBM_PEAK_GBS})
        else:
            fl = 2.0 * M * cfg.N * cfg.K
            out.append({"workload": f"prefill M={M}, codes in the slab-tile layout (lords_repack)", "us_per_launch": us, "launch_mode": mode,
                        "value": fl / us / 1e6, "unit": "TFLOP/s", "frac_of_mfma_peak": fl / us / 1e6 / MFMA_BF16_PEAK_TFLOPS})
        del tiled, X, Y
    return out


BLOCK_SHAPES = {"q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
                "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336)}


def make_blocks(bits, li, torch, L, seed0):
    """Enough Llama-3-8B-shaped blocks (seven linear layers each, rank 32) at one code width that no launch
    finds its weights in the last-level cache.  Returns (blocks, activations by width, codebook, bytes of codes)."""
    per_block = sum(n * k for n, k in BLOCK_SHAPES.values()) * bits // 8
    nblocks = int(-(-COLD_BYTES // per_block))
    blocks, xs, codebook = [], {}, None
    for b in range(nblocks):
        layers = {}
        for j, (name, (n, k)) in enumerate(BLOCK_SHAPES.items()):
            cs = li.make_case("qproj_4b", M=2, N=n, K=k, bits=bits, seed=seed0 + 7 * b + j)
            xs.setdefault(k, L.bf16_from_bits(cs.X_bf16))
            layers[name] = (torch.from_numpy(cs.codes).cuda(), L.bf16_from_bits(cs.B_bf16), L.bf16_from_bits(cs.A_bf16))
            codebook = torch.from_numpy(cs.codebook.copy()).cuda()
        blocks.append(layers)
    return blocks, xs, codebook, per_block


def run_block(L, ly, codebook, bits, M, X4, X14, outs, r=32):
    """The seven linear layers of one block as four calls: q/k/v in one launch, o, gate/up with its activation, down."""
    K0, I = 4096, 14336
    Yq, Yk, Yv, Yo, H, Yd = outs
    q, k, v = ly["q"], ly["k"], ly["v"]
    L.lords_matmul_batched(X4, [q[0], k[0], v[0]], codebook, [q[1], k[1], v[1]], [q[2], k[2], v[2]],
                           [Yq, Yk, Yv], [4096, 1024, 1024], M, K0, r, bits)
    o = ly["o"]
    L.lords_matmul(X4, o[0], codebook, o[1], o[2], Yo, M, 4096, K0, r, bits)
    g, u = ly["gate"], ly["up"]
    L.lords_gate_up(X4, g[0], g[1], g[2], u[0], u[1], u[2], codebook, H, M, I, K0, r, bits)
    d = ly["down"]
    L.lords_matmul(X14, d[0], codebook, d[1], d[2], Yd, M, K0, I, r, bits)


def block_outputs(M, torch):
    f32 = dict(dtype=torch.float32, device="cuda")
    return (torch.zeros((M, 4096), **f32), torch.zeros((M, 1024), **f32), torch.zeros((M, 1024), **f32),
            torch.zeros((M, 4096), **f32), torch.zeros((M, 14336), **f32), torch.zeros((M, 4096), **f32))


def bench_block(args, L, li, torch):
    """Context figures.  (1) The seven linear layers of one Llama-3-8B-shaped block at one token and at two, as
    four calls, 4-bit codes of rank 32, rotating through enough blocks that no launch finds its weights in the
    last-level cache.  (2) A 32-block stack at one token under the mixed-precision schedules of the paper's
    ultra-low-bit setting (4-bit levels in the first 1/2, 1/4, 1/8 of the blocks, 2-bit levels in the rest:
    3, 2.5 and 2.25 bits on average), widths from lords_mixed_schedule, beside the uniform 4-bit stack."""
    bits, r = 4, 32
    blocks, xs, codebook, per_block = make_blocks(bits, li, torch, L, 5000)
    nblocks = len(blocks)
    X4, X14 = xs[4096], xs[14336]        # stand-ins for the activations that feed each layer (shapes only)
    out = []
    for M in (1, 2):
        outs = block_outputs(M, torch)

        def step(i):
            run_block(L, blocks[i % nblocks], codebook, bits, M, X4, X14, outs, r)

        _, ev_ms, mode, _ = time_steps(step, 60, 6, torch, use_graph=not args.no_graph)
        us = ev_ms * 1e3 / 60
        out.append({"workload": f"decode M={M}, the seven linear layers of one Llama-3-8B-shaped block in four calls "
                                f"(4-bit, rank 32; {nblocks} rotating blocks)",
                    "us_per_step": us, "launch_mode": mode, "value": per_block / us / 1e3, "unit": "GB/s (codes only)",
                    "frac_of_hbm_peak": per_block / us / 1e3 / HBM_PEAK_GBS,
                    "ms_for_32_blocks": us * 32 / 1e3})

    # (2) mixed-precision stacks
    blocks2, _, codebook2, per_block2 = make_blocks(2, li, torch, L, 7000)
    pools = {4: (blocks, codebook, per_block), 2: (blocks2, codebook2, per_block2)}
    outs = block_outputs(1, torch)
    n_layers = 32
    base_ms = None
    for label, fraction in (("4", 1.0), ("3", 0.5), ("2.5", 0.25), ("2.25", 0.125)):
        widths, avg = L.lords_mixed_schedule(n_layers, fraction, 4, 2)

        def step(i, widths=widths):
            seen = {4: 0, 2: 0}
            for w in widths:
                pool, cb, _ = pools[w]
                run_block(L, pool[(i * n_layers + seen[w]) % len(pool)], cb, w, 1, X4, X14, outs, r)
                seen[w] += 1

        _, ev_ms, mode, _ = time_steps(step, 8, 2, torch, use_graph=not args.no_graph)
        ms = ev_ms / 8
        nbytes = sum(pools[w][2] for w in widths)
        if base_ms is None:
            base_ms = ms
        out.append({"workload": f"decode M=1, 32-block stack (224 linear layers, rank 32), {label} bits on average "
                                f"({widths.count(4)} blocks at 4 bits, then {widths.count(2)} at 2 bits)",
                    "average_bits": avg, "ms_per_token": ms, "launch_mode": mode, "value": nbytes / ms / 1e6,
                    "unit": "GB/s (codes only)", "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS,
                    "speedup_over_4_bits": base_ms / ms})
    return out


def bench_backward(args, L, li, torch):
    """Context figures for one fine-tuning step of the scale factors on the headline layer, 2048 tokens:
    forward, gradient with respect to the activations (through the transposed codes), gradients with
    respect to B and A."""
    name, M = "gateup_4b", 2048
    cfg = li.CONFIGS[name]
    cs, sets, X, codebook = make_sets(name, M, 1, li, torch)
    codes, B, A = sets[0]
    dY = L.bf16_from_bits(li.make_output_grad(M, cfg.N, 4000)[0])
    codes_t = torch.empty((cfg.K, cfg.N * cfg.bits // 8), dtype=torch.uint8, device="cuda")
    L.lords_transpose_codes(codes, codes_t, cfg.N, cfg.K, cfg.bits)
    Y = torch.zeros((M, cfg.N), dtype=torch.bfloat16, device="cuda")
    dX = torch.zeros((M, cfg.K), dtype=torch.bfloat16, device="cuda")
    dB = torch.zeros((cfg.N, cfg.r), dtype=torch.float32, device="cuda")
    dA = torch.zeros((cfg.r, cfg.K), dtype=torch.float32, device="cuda")
    legs = {
        "forward": lambda i: L.lords_matmul(X, codes, codebook, B, A, Y, M, cfg.N, cfg.K, cfg.r, cfg.bits),
        "backward_input": lambda i: L.lords_backward_input(dY, codes_t, codebook, B, A, dX, M, cfg.N, cfg.K, cfg.r, cfg.bits),
        "backward_factors": lambda i: L.lords_backward_factors(dY, X, codes, codebook, B, A, dB, dA, M, cfg.N, cfg.K, cfg.r,
                                                               cfg.bits),
    }
    fl = 2.0 * M * cfg.N * cfg.K
    res = {}
    for label, fn in legs.items():
        _, ev_ms, _, _ = time_steps(fn, 10, 3, torch, use_graph=False)
        res[label] = ev_ms * 1e3 / 10
    total = sum(res.values())
    return [{"workload": f"fine-tuning step of the scale factors, M={M} on the headline layer: forward + dX + (dB, dA)",
             "us_per_step": total, "us_by_leg": res, "value": 3 * fl / total / 1e6, "unit": "TFLOP/s",
             "frac_of_mfma_peak": 3 * fl / total / 1e6 / MFMA_BF16_PEAK_TFLOPS}]


def bench_shared_input(args, L, li, torch):
    """Context figures for the decode calls that serve several matrices reading the same activations:
    query/key/value of the Llama-3-8B block in one launch, and its gate/up pair with silu(gate)*up on the
    way out, each beside the same matrices served by separate lords_matmul calls; one token and two."""
    out = []
    bf16_tensor = L.bf16_from_bits
    # ---- q/k/v: 4096, 1024, 1024 rows of 4096 columns, 4 bits, rank 32
    cfg = li.CONFIGS["qproj_4b"]
    Ns = (4096, 1024, 1024)
    per_set = sum(Ns) * cfg.K * cfg.bits // 8
    nsets = int(-(-COLD_BYTES // per_set))
    sets, cs0 = [], None
    for s in range(nsets):
        layers = []
        for j, N in enumerate(Ns):
            cs = li.make_case("qproj_4b", M=2, N=N, seed=3000 + 3 * s + j)
            cs0 = cs0 or cs
            layers.append((torch.from_numpy(cs.codes).cuda(), bf16_tensor(cs.B_bf16), bf16_tensor(cs.A_bf16)))
        sets.append(layers)
    X = bf16_tensor(cs0.X_bf16)
    codebook = torch.from_numpy(cs0.codebook.copy()).cuda()
    for M in (1, 2):
        Ys = [torch.zeros((M, N), dtype=torch.float32, device="cuda") for N in Ns]

        def one_launch(i):
            ls = sets[i % nsets]
            L.lords_matmul_batched(X, [l[0] for l in ls], codebook, [l[1] for l in ls], [l[2] for l in ls], Ys, Ns,
                                   M, cfg.K, cfg.r, cfg.bits)

        def separate(i):
            for (codes, B, A), Y, N in zip(sets[i % nsets], Ys, Ns):
                L.lords_matmul(X, codes, codebook, B, A, Y, M, N, cfg.K, cfg.r, cfg.bits)

        ab = sum(algorithmic_bytes(M, N, cfg.K, cfg.r, cfg.bits) for N in Ns) - 2 * M * cfg.K * 2
        res = {}
        for label, fn in (("one_launch", one_launch), ("separate_calls", separate)):
            _, ev_ms, _, _ = time_steps(fn, 100, 5, torch, use_graph=not args.no_graph)
            res[label] = ev_ms * 1e3 / 100
        out.append({"workload": f"decode M={M}, q/k/v (4096+1024+1024 x 4096, 4-bit, rank 32) sharing X",
                    "us_per_step": res["one_launch"], "us_per_step_separate_calls": res["separate_calls"],
                    "value": ab / res["one_launch"] / 1e3, "unit": "GB/s",
                    "frac_of_hbm_peak": ab / res["one_launch"] / 1e3 / HBM_PEAK_GBS})
    del sets, Ys

    # ---- gate/up pair of the headline layer shape, H = silu(gate) * up
    cfg = li.CONFIGS["gateup_4b"]
    per_set = 2 * cfg.N * cfg.K * cfg.bits // 8
    nsets = int(-(-COLD_BYTES // per_set))
    _, layers, X, codebook = make_sets("gateup_4b", 2, 2 * nsets, li, torch)
    for M in (1, 2):
        H = torch.zeros((M, cfg.N), dtype=torch.float32, device="cuda")
        G, U = torch.zeros_like(H), torch.zeros_like(H)

        def fused(i):
            (cg, Bg, Ag), (cu, Bu, Au) = layers[2 * (i % nsets)], layers[2 * (i % nsets) + 1]
            L.lords_gate_up(X, cg, Bg, Ag, cu, Bu, Au, codebook, H, M, cfg.N, cfg.K, cfg.r, cfg.bits)

        def two_calls(i):
            (cg, Bg, Ag), (cu, Bu, Au) = layers[2 * (i % nsets)], layers[2 * (i % nsets) + 1]
            L.lords_matmul(X, cg, codebook, Bg, Ag, G, M, cfg.N, cfg.K, cfg.r, cfg.bits)
            L.lords_matmul(X, cu, codebook, Bu, Au, U, M, cfg.N, cfg.K, cfg.r, cfg.bits)

        ab = 2 * algorithmic_bytes(M, cfg.N, cfg.K, cfg.r, cfg.bits) - M * cfg.K * 2 - M * cfg.N * 4
        res = {}
        for label, fn in (("one_launch", fused), ("two_products", two_calls)):
            _, ev_ms, _, _ = time_steps(fn, 100, 5, torch, use_graph=not args.no_graph)
            res[label] = ev_ms * 1e3 / 100
        out.append({"workload": f"decode M={M}, gate/up pair (2 x 14336 x 4096, 4-bit, rank 32), H = silu(gate)*up",
                    "us_per_step": res["one_launch"],
                    "us_per_step_two_products_without_the_activation": res["two_products"],
                    "value": ab / res["one_launch"] / 1e3, "unit": "GB/s",
                    "frac_of_hbm_peak": ab / res["one_launch"] / 1e3 / HBM_PEAK_GBS})
    return out


def gpu_sets(N, K, bits, r, M, nsets, torch, seed):
    """Weight sets drawn on the GPU (the same distributions as lords_inputs.make_case: uniform code bytes, A ~ U(0.5, 1.5),
    B ~ U(0.5, 1.5) * 0.02 / r, X ~ N(0, 1), all bf16): the extra legs below need no bit-identical CPU copy."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    sets = []
    for _ in range(nsets):
        codes = torch.randint(0, 256, (N, K * bits // 8), dtype=torch.uint8, device="cuda", generator=g)
        B = ((torch.rand((N, r), device="cuda", generator=g) + 0.5) * (0.02 / r)).to(torch.bfloat16)
        A = (torch.rand((r, K), device="cuda", generator=g) + 0.5).to(torch.bfloat16)
        sets.append((codes, B, A))
    X = torch.randn((M, K), device="cuda", generator=g).to(torch.bfloat16)
    return sets, X


# the layer shapes the method is quoted on, beside the headline layer: (label, N, K, bits, rank, token counts)
CONFIG_LEGS = [
    ("Llama-3-8B q_proj 4096x4096, 4-bit, rank 32", 4096, 4096, 4, 32, (1, 4, 16)),
    ("Llama-3-8B gate/up 14336x4096, 3-bit, rank 48", 14336, 4096, 3, 48, (1, 16)),
    ("Llama-3-8B down 4096x14336, 3-bit, rank 48", 4096, 14336, 3, 48, (1, 16)),
    ("Llama-3-8B down 4096x14336, 4-bit, rank 32", 4096, 14336, 4, 32, (1, 2048)),
    ("Llama-3-8B gate/up 14336x4096, 4-bit, rank 32", 14336, 4096, 4, 32, (2,)),
    ("Llama-3-70B-shaped 28672x8192, 2-bit, rank 64", 28672, 8192, 2, 64, (1, 16, 256, 4096)),
]


def bench_configs(args, L, li, torch, ceilings):
    """Every other layer shape and token count the method is quoted on: decode legs (M <= 16) against the HBM line
    (and, where the scale regeneration 2rNK outweighs the bytes, against the MFMA line as well: the larger of the
    two times is the bound), prefill legs against the bf16 MFMA line.  Rotating weight sets as for the headline."""
    import itertools
    codebooks = {b: torch.from_numpy(li.nf_codebook(b).copy()).cuda() for b in (2, 3, 4)}
    out = []
    for (label, N, K, bits, r, Ms), seed in zip(CONFIG_LEGS, itertools.count(9000)):
        per_set = N * K * bits // 8
        for M in Ms:
            decode = M <= 16
            nsets = int(-(-COLD_BYTES // per_set)) if decode else 2
            sets, X = gpu_sets(N, K, bits, r, M, nsets, torch, seed)
            Y = torch.zeros((M, N), dtype=torch.float32 if decode else torch.bfloat16, device="cuda")

            def run_step(i):
                codes, B, A = sets[i % nsets]
                L.lords_matmul(X, codes, codebooks[bits], B, A, Y, M, N, K, r, bits)

            steps = 100 if decode else (10 if M * N * K < 3e11 else 4)
            _, ev_ms, mode, _ = time_steps(run_step, steps, 5, torch, use_graph=not args.no_graph)
            us = ev_ms * 1e3 / steps
            leg = {"workload": f"{'decode' if decode else 'prefill'} M={M}, {label}", "us_per_launch": us, "launch_mode": mode}
            if decode:
                ab = algorithmic_bytes(M, N, K, r, bits)
                t_hbm = ab / HBM_PEAK_GBS / 1e3                      # us
                t_mfma = 2.0 * r * N * K / MFMA_BF16_PEAK_TFLOPS / 1e6   # us: the scale contraction alone
                leg.update({"value": ab / us / 1e3, "unit": "GB/s", "frac_of_hbm_peak": ab / us / 1e3 / HBM_PEAK_GBS,
                            "frac_of_measured_read": ab / us / 1e3 / ceilings["stream_read_GBs"] if ceilings else None,
                            "us_at_hbm_peak": t_hbm, "us_of_scale_contraction_at_mfma_peak": t_mfma,
                            "binding_line": "mfma (scale contraction)" if t_mfma > t_hbm else "hbm",
                            "frac_of_binding_line": max(t_hbm, t_mfma) / us})
            else:
                fl = 2.0 * M * N * K
                leg.update({"value": fl / us / 1e6, "unit": "TFLOP/s", "frac_of_mfma_peak": fl / us / 1e6 / MFMA_BF16_PEAK_TFLOPS,
                            "frac_of_measured_mfma": fl / us / 1e6 / ceilings["mfma_bf16_TFLOPs"] if ceilings else None})
            out.append(leg)
            del sets, X, Y
    return out


def bench_ceilings(args, L, torch):
    """What this GPU gives to a kernel that does nothing else: (a) a read-only pass over a cold 30 MB buffer per launch
    (21 buffers in rotation: the headline layer's footprint and launch pattern), (b) over one 640 MB buffer per launch,
    (c) register-resident bf16 MFMA chains.  HIP-graph replays, like the legs they are quoted beside."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    small = [torch.randint(0, 255, (30 << 20,), dtype=torch.uint8, device="cuda") for _ in range(21)]
    _, ev_ms, _, _ = time_steps(lambda i: L.lords_probe_stream_read(small[i % 21], sink), 210, 21, torch, use_graph=not args.no_graph)
    us_small = ev_ms * 1e3 / 210
    del small
    big = torch.randint(0, 255, (640 << 20,), dtype=torch.uint8, device="cuda")
    _, ev_ms, _, _ = time_steps(lambda i: L.lords_probe_stream_read(big, sink), 10, 2, torch, use_graph=not args.no_graph)
    us_big = ev_ms * 1e3 / 10
    del big
    rates = {}
    for pattern in (0, 1):
        flop = L.lords_probe_mfma_bf16(20000, sink, pattern)
        _, ev_ms, _, _ = time_steps(lambda i: L.lords_probe_mfma_bf16(20000, sink, pattern), 10, 2, torch, use_graph=not args.no_graph)
        rates[pattern] = flop / (ev_ms * 1e3 / 10) / 1e6
    return {"cold_30MB_read_us_per_launch": us_small, "cold_30MB_read_GBs": (30 << 20) / us_small / 1e3,
            "stream_read_GBs": (640 << 20) / us_big / 1e3,
            "mfma_bf16_TFLOPs": rates[1], "mfma_bf16_TFLOPs_trivial_operands": rates[0],
            "note": "read-only pass with 16-byte loads (lords_probe_stream_read); eight independent v_mfma_f32_16x16x32_bf16 "
                    "chains per wave, operands in registers (lords_probe_mfma_bf16): with operands that differ in every lane "
                    "and element (the ceiling the GEMM is quoted against: its operands are real data), and with operands of "
                    "ones and small integers (few bits toggling: the chip holds a higher clock)"}


def cpu_baseline(li, ab):
    """The fp64 C oracle, as it stands, on the decode workload (M = 1, whole layer), host cores."""
    from oracle import lords_oracle_c as oc
    cs = li.make_case("gateup_4b", M=1, seed=1000)
    threads = oc.threads()
    oc.matmul(cs.X_f32, cs.codes[:256], cs.codebook, cs.B_f32[:256], cs.A_f32, cs.bits)     # warm-up, small slab
    reps, t_total = 0, 0.0
    while reps < 3 or (t_total < 2.0 and reps < 20):
        t0 = time.perf_counter()
        oc.matmul(cs.X_f32, cs.codes, cs.codebook, cs.B_f32, cs.A_f32, cs.bits)
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    return {"value": ab / sec / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{reps} passes of the whole decode layer (M=1, N=14336, K=4096, 4-bit, r=32) through the "
                      f"plain-C fp64 oracle with OpenMP over rows; {sec * 1e3:.1f} ms per pass",
            "ms_per_step": sec * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed repetitions of the timed work for this long before each timed region (clock ramp)")
    ap.add_argument("--workload", choices=["decode", "prefill", "shared_input", "backward", "configs", "ceilings", "all"], default="all",
                    help="decode / prefill: the headline workloads; shared_input, backward: context figures only "
                         "(profiling runs); all: everything")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads and writes 256 MiB each (the known-size "
                         "reference for scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    globals()["SETTLE_MS"] = max(0.0, args.settle_ms)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives are part of it)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import lords_inputs as li
    import paper_2601_22716_amd as L
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    L.library()      # fail loudly if liblords.so is missing: there is no fallback

    line = {"metric": "decode GB/s (algorithmic bytes / time, M=1)", "value": None, "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": None, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "clock_settle_ms": args.settle_ms,
            "clock_settle_note": "each timed region follows untimed repetitions of the same work for clock_settle_ms: "
                                 "the clocks of an idle GPU take tens of milliseconds of load to come up"}
    ab = algorithmic_bytes(1, 14336, 4096, 32, 4)
    ceilings = None
    if args.workload in ("ceilings", "configs", "all") and not args.calibrate_copy:
        ceilings = bench_ceilings(args, L, torch)
        line["measured_ceilings"] = ceilings
    if args.workload in ("decode", "all"):
        d, *_ = bench_decode(args, L, li, torch)
        if ceilings:
            d["roofline"]["measured_peak"] = ceilings["stream_read_GBs"]
            d["roofline"]["frac_of_measured"] = d["roofline"]["achieved"] / ceilings["stream_read_GBs"]
            d["roofline"]["frac_of_measured_cold_30MB_read"] = d["roofline"]["achieved"] / ceilings["cold_30MB_read_GBs"] \
                * (30 << 20) / ab
        line.update(d)
    if args.workload in ("prefill", "all"):
        p = bench_prefill(args, L, li, torch)
        if ceilings:
            p["roofline"]["measured_peak"] = ceilings["mfma_bf16_TFLOPs"]
            p["roofline"]["frac_of_measured"] = p["roofline"]["achieved"] / ceilings["mfma_bf16_TFLOPs"]
        if args.workload == "prefill":
            line.update({k: p[k] for k in ("metric", "value", "unit", "steps", "ms_per_step", "config", "roofline")})
        else:
            line["prefill"] = p
    if args.workload == "all" and not args.calibrate_copy:
        line["other_workloads"] = bench_other(args, L, li, torch) + bench_configs(args, L, li, torch, ceilings)
    if args.workload == "configs":
        line["other_workloads"] = bench_configs(args, L, li, torch, ceilings)
    if args.workload == "shared_input":
        line["other_workloads"] = bench_shared_input(args, L, li, torch) + bench_block(args, L, li, torch)
    if args.workload == "backward":
        line["other_workloads"] = bench_backward(args, L, li, torch)
    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        line["calibration"] = {"kernel": "torch elementwise add, fp32", "read_bytes": src.numel() * 4,
                               "write_bytes": dst.numel() * 4, "launches": 3}
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(li, ab)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
