#!/usr/bin/env python3
"""Benchmark of the Axe-layout hot path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the GEMM hot path (host layout analysis, HBM -> LDS -> VGPR -> MFMA -> HBM)
over one batch of synthetic input: the bf16 GEMM M = N = K = 8192 (configuration 3), inputs
resident in HBM, rotating over two buffer sets.  The headline value is its whole-job TFLOP/s.
The same JSON line carries, under "companions", the other configurations measured in the same
run (relayout GB/s, fp8 GEMM, the tensor-parallel shard, the 256^3 GEMM, layout evaluation, and
for context the measured ceilings: register-only MFMA loops and a plain device copy), the roofline
of the dominant kernel and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16": 2516.6, "fp8": 5033.2, "hbm": 8000.0}     # TFLOP/s, TFLOP/s, GB/s (MI355X, dense)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


MIN_WARM_MS = 40.0        # companions: see time_loop


def settle(fn, max_ms=400.0, window=8, tol=0.015):
    """Launches fn until its per-launch device time has stopped falling: after the host has been busy (generating
    inputs) the GPU's clocks take a while to come up, and a timed region that starts inside that ramp measures
    the ramp (the same 0.73 ms kernel reads 0.86 ms in the first 20 ms).  Stops when the means of two consecutive windows of
    `window` launches agree within `tol`, or after max_ms.  Returns what it did, for the JSON line: it is extra
    untimed warm-up, before the `--warmup` steps, and does no part of the timed work."""
    import torch
    t0 = time.perf_counter()
    prev, n, hist = None, 0, []
    while (time.perf_counter() - t0) * 1e3 < max_ms:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(window + 1)]
        evs[0].record()
        for k in range(window):
            fn(n + k)
            evs[k + 1].record()
        torch.cuda.synchronize()
        n += window
        cur = sum(evs[k].elapsed_time(evs[k + 1]) for k in range(window)) / window
        hist.append(cur)
        if prev is not None and abs(cur - prev) <= tol * prev:
            break
        prev = cur
    return {"launches": n, "ms": (time.perf_counter() - t0) * 1e3, "first_window_kernel_ms": hist[0], "last_window_kernel_ms": hist[-1]}


def per_launch(fn, steps):
    """Device time of each of `steps` launches (one event pair per launch), after the timed region."""
    import torch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record()
    for k in range(steps):
        fn(k)
        evs[k + 1].record()
    torch.cuda.synchronize()
    return sorted(evs[k].elapsed_time(evs[k + 1]) for k in range(steps))


def time_loop(fn, steps, warmup, min_warm_ms=None):
    """Returns (wall ms per step, device ms per step from HIP events on the launch stream).
    After the host has been busy for a while (generating inputs) the first 10 - 20 ms of GPU work run at lower
    clocks (measured: a 0.2 ms kernel timed after 20 warm-up launches reads 10 % slower than after 200).  The
    headline step is brought to a steady clock by settle() and then does exactly `warmup` untimed steps; the
    companion kernels keep warming up until min_warm_ms have passed."""
    import torch
    min_warm_ms = MIN_WARM_MS if min_warm_ms is None else min_warm_ms
    t_w = time.perf_counter()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    i = warmup
    while (time.perf_counter() - t_w) * 1e3 < min_warm_ms:
        for _ in range(max(1, warmup)):
            fn(i)
            i += 1
        torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        fn(i)
    ev1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, ev0.elapsed_time(ev1) / steps


def dev(a):
    import torch
    a = np.ascontiguousarray(a)
    view = {1: np.uint8, 2: np.int16, 4: np.int32}[a.dtype.itemsize]
    return torch.from_numpy(a.view(view)).cuda()


def gemm_setup(g, n_sets, device_axis=False, tile=0, scale_a_rows=0):
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    As, Bs, Cs = W.gemm_specs(g, device_axis=device_axis, shard=3)
    axes = ["m", "gpuid"]
    out_t = torch.float32 if g.out_dtype == "f32" else torch.int16
    sets = []
    for s in range(n_sets):
        dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
        if s:                       # other sets: same statistics, different bits (rotated rows)
            dA, dB = torch.roll(dA, 4096 * s), torch.roll(dB, 4096 * s)
        dC = torch.zeros(g.M * g.N, dtype=out_t, device="cuda")
        sets.append((dA, dB, dC))
    sa = torch.from_numpy(g.scale_a).cuda() if g.scale_a is not None else None
    sb = torch.from_numpy(g.scale_b).cuda() if g.scale_b is not None else None
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16 if g.dtype == "bf16" else B.AXE_FP8_E4M3,
                      B.AXE_F32 if g.out_dtype == "f32" else B.AXE_BF16,
                      B.Layout(As, axes), B.Layout(Bs, axes), B.Layout(Cs, axes),
                      g.M * g.K, g.N * g.K, g.M * g.N, sa, sb, tile_hint=tile,
                      scale_dtype=B.AXE_SCALE_E8M0 if g.scale_dtype == "e8m0" else B.AXE_SCALE_F32, scale_a_rows=scale_a_rows)
    def step(i):
        dA, dB, dC = sets[i % n_sets]
        B.axe_gemm(desc, dA, dB, dC)
    return step, sets, desc


def bench_gemm(name, g, steps, warmup, n_sets=2, device_axis=False, min_warm_ms=None, headline=False, scale_a_rows=0):
    step, sets, desc = gemm_setup(g, n_sets, device_axis, scale_a_rows=scale_a_rows)
    st = settle(step) if headline else None
    wall, devms = time_loop(step, steps, warmup, min_warm_ms)
    flops = 2.0 * g.M * g.N * g.K
    r = {"workload": name, "ms_per_step": wall, "kernel_ms": devms, "tflops": flops / (wall * 1e-3) / 1e12,
         "kernel_tflops": flops / (devms * 1e-3) / 1e12}
    r["frac_of_peak"] = r["kernel_tflops"] / PEAK["fp8" if g.dtype == "fp8" else "bf16"]
    if headline:
        pl = per_launch(step, steps)
        r["settle"] = st
        r["per_launch_kernel_ms"] = {"min": pl[0], "median": pl[len(pl) // 2], "max": pl[-1]}
        log(f"[bench] {name}: clocks settled after {st['launches']} untimed launches ({st['ms']:.0f} ms; per launch "
            f"{st['first_window_kernel_ms']:.4f} -> {st['last_window_kernel_ms']:.4f} ms); per-launch times after the timed region: "
            f"min {pl[0]:.4f} median {pl[len(pl) // 2]:.4f} max {pl[-1]:.4f} ms")
    log(f"[bench] {name}: {wall:.4f} ms/step wall, {devms:.4f} ms device, {r['kernel_tflops']:.1f} TFLOP/s "
        f"({100 * r['frac_of_peak']:.1f}% of peak)")
    return r, sets


def graph_replay_us(step, launches=64, replays=30):
    """Device microseconds per launch when `launches` calls of step() are recorded into one HIP graph and the graph
    is replayed: what a launch-bound loop costs once the host is out of it.  The library allocates nothing and
    records no memset, so its launches can be captured as they are."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(0)                                                     # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(launches):
            step(i)
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(replays):
        graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) * 1e3 / (replays * launches)


def bench_relayout(steps, warmup, n_pairs=4):
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    rows = cols = 8192
    words = W.config2("uniform")
    Ls, Ld = B.Layout(W.row_major_spec(rows, cols)), B.Layout(W.blocked_swizzled_spec(rows, cols))
    pairs = []
    for p in range(n_pairs):
        src = dev(words.reshape(-1))
        if p:
            src = torch.roll(src, 777 * p)
        pairs.append((src, torch.zeros(rows * cols, dtype=torch.int16, device="cuda")))
    nbytes = 2.0 * rows * cols * 2          # read + write
    # one plain device copy of the same 128 MiB (untimed): the known-size kernel against which the
    # FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this script are calibrated
    pairs[0][1].copy_(pairs[0][0])
    out = {}
    for label, np_ in (("rotating", n_pairs), ("single_pair", 1)):
        def step(i, np_=np_):
            s, d = pairs[i % np_]
            B.axe_relayout(Ls, Ld, (rows, cols), s, d)
        wall, devms = time_loop(step, steps, warmup)
        out[label] = {"ms_per_step": wall, "kernel_ms": devms, "GBps": nbytes / (devms * 1e-3) / 1e9}
    def back(i):
        s, d = pairs[i % n_pairs]
        B.axe_relayout(Ld, Ls, (rows, cols), d, s)
    wall, devms = time_loop(back, steps, warmup)
    out["inverse_rotating"] = {"ms_per_step": wall, "kernel_ms": devms, "GBps": nbytes / (devms * 1e-3) / 1e9}
    out["frac_of_hbm_peak"] = out["rotating"]["GBps"] / PEAK["hbm"]
    log(f"[bench] relayout 8192^2 bf16 -> 128x64 swizzled tiles: {out['rotating']['GBps']:.0f} GB/s rotating "
        f"({100 * out['frac_of_hbm_peak']:.1f}% of HBM peak), {out['single_pair']['GBps']:.0f} GB/s single pair, "
        f"inverse {out['inverse_rotating']['GBps']:.0f} GB/s")
    return out


def bench_transpose(steps, warmup, n_pairs=4):
    """Row-major -> column-major of the same 8192 x 8192 bf16 matrix: source and destination are
    contiguous along different digits, the relayout goes through LDS tiles."""
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    rows = cols = 8192
    Ls, Ld = B.Layout(W.row_major_spec(rows, cols)), B.Layout(W.col_major_spec(rows, cols))
    pairs = [(torch.randint(-30000, 30000, (rows * cols,), dtype=torch.int16, device="cuda"),
              torch.zeros(rows * cols, dtype=torch.int16, device="cuda")) for _ in range(n_pairs)]
    wall, devms = time_loop(lambda i: B.axe_relayout(Ls, Ld, (rows, cols), *pairs[i % n_pairs]), steps, warmup)
    assert torch.equal(pairs[0][1].view(cols, rows), pairs[0][0].view(rows, cols).t())
    r = {"ms_per_step": wall, "kernel_ms": devms, "GBps": 2.0 * rows * cols * 2 / (devms * 1e-3) / 1e9}
    r["frac_of_hbm_peak"] = r["GBps"] / PEAK["hbm"]
    log(f"[bench] relayout 8192^2 bf16 row-major -> column-major (transposing tiles): {r['GBps']:.0f} GB/s rotating "
        f"({100 * r['frac_of_hbm_peak']:.1f}% of HBM peak)")
    del pairs
    # the same with extents that are no multiples of a 16-byte chunk: the element-wise tiles
    ro, co = 8191, 8193
    Ls, Ld = B.Layout(W.row_major_spec(ro, co)), B.Layout(W.col_major_spec(ro, co))
    pairs = [(torch.randint(-30000, 30000, (ro * co,), dtype=torch.int16, device="cuda"),
              torch.zeros(ro * co, dtype=torch.int16, device="cuda")) for _ in range(n_pairs)]
    _, d_odd = time_loop(lambda i: B.axe_relayout(Ls, Ld, (ro, co), *pairs[i % n_pairs]), steps, warmup)
    assert torch.equal(pairs[0][1].view(co, ro), pairs[0][0].view(ro, co).t())
    r["odd_extents_8191x8193"] = {"kernel_ms": d_odd, "GBps": 2.0 * ro * co * 2 / (d_odd * 1e-3) / 1e9}
    del pairs
    # a register layout as destination: the A operand layout of the 256 x 256 kernel (axe_gemm_describe), tiled over the
    # matrix (axe_layout_tile) and folded onto memory as [tile][wave][lane][reg] (axe_layout_flatten); both wave copies
    M = K = 8192
    desc = B.GemmDesc(M, 256, K, B.AXE_BF16, B.AXE_BF16, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, 256)),
                      B.Layout(W.row_major_spec(M, 256)), M * K, 256 * K, M * 256, tile_hint=B.AXE_TILE_256x256x64)
    axes = ["m", "lds", "wg", "wave", "lane", "reg"]
    spec, tshape = B.axe_gemm_describe(desc, B.AXE_DESC_A_OPERAND)
    gm, gk = M // tshape[0], K // tshape[1]
    tiled, shape = B.layout_tile(B.Layout(W.spec([(gm, gk, "wg"), (gk, 1, "wg")]), axes), (gm, gk), B.Layout(spec, axes), tshape)
    span = B.layout_span(B.Layout(tiled, axes))
    regs = span["reg"]
    dstL = B.Layout(B.layout_flatten(B.Layout(tiled, axes), {"reg": 1, "lane": regs, "wave": span["lane"] * regs,
                                                               "wg": span["wave"] * span["lane"] * regs}, "m"), axes)
    srcL = B.Layout(W.spec([(gm, tshape[0] * K, "m"), (tshape[0], K, "m"), (gk, tshape[1], "m"), (tshape[1], 1, "m")]), axes)
    n_dst = gm * gk * span["wave"] * span["lane"] * regs
    a = torch.randint(-30000, 30000, (M * K,), dtype=torch.int16, device="cuda")
    outs = [torch.zeros(n_dst, dtype=torch.int16, device="cuda") for _ in range(2)]
    _, d_reg = time_loop(lambda i: B.axe_relayout(srcL, dstL, shape, a, outs[i % 2]), steps, warmup)
    r["to_mfma_operand_registers_8192"] = {"kernel_ms": d_reg, "replicas": n_dst // (M * K),
                                           "GBps": (M * K + n_dst) * 2.0 / (d_reg * 1e-3) / 1e9}
    log(f"[bench] relayout 8191 x 8193 bf16 row-major -> column-major (element-wise tiles): {r['odd_extents_8191x8193']['GBps']:.0f} GB/s; "
        f"8192^2 bf16 -> MFMA operand register order, both wave copies: {r['to_mfma_operand_registers_8192']['GBps']:.0f} GB/s (read + written)")
    return r


def bench_grouped(steps, warmup, dtype="f16", sweep=(1, 8, 64, 256, 512, 2048, 4096)):
    """The expert computation of an MoE layer (hidden 2048, expert intermediate 768, 128 experts, 8 per token), in fp16
    like the paper's layer: gemm1 (gate and up projections, gated activation fused) and gemm2 (down projection) as
    grouped GEMMs over the routed rows sorted by expert, offsets on the device, over a sweep of token counts as in the
    paper's figure.  Weights are packed once by axe_relayout (untimed, as a server would do at load time) into
    contiguous 256 x 64 blocks, gate and up rows interleaved for gemm1.  At the largest count gemm1 and gemm2 are also
    timed without the epilogue on plain and on blocked weights."""
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    dt = B.AXE_F16 if dtype == "f16" else B.AXE_BF16
    top = max(sweep)
    full = {"gemm1": W.moe_gemm1(top, dtype=dtype), "gemm2": W.moe_gemm2(top, dtype=dtype)}
    out = {"experts": W.MOE_EXPERTS, "experts_per_token": W.MOE_TOPK, "dtype": dtype, "sweep": {}}
    layer = {t: 0.0 for t in sweep}
    packed = {}
    for name, f in full.items():
        gated = name == "gemm1"
        NC = f.N // 2 if gated else f.N
        plainL = B.Layout(W.grouped_gemm_specs(f)[1])
        blkL = B.Layout(W.blocked_b_spec(f.K, f.N, G=f.G))
        useL = B.Layout(W.gated_b_spec(f.K, f.N, f.G, True)) if gated else blkL
        dB = dev(f.b_gnk.reshape(-1))
        dBblk, dBuse = torch.empty_like(dB), None
        B.axe_relayout(plainL, blkL, (f.G, f.K, f.N), dB, dBblk)
        if gated:
            dBuse = torch.empty_like(dB)
            B.axe_relayout(plainL, useL, (f.G, f.K, f.N), dB, dBuse)
        else:
            dBuse = dBblk
        for tokens in sweep:
            rows = W.moe_group_rows(tokens, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
            M = int(rows[-1])
            dA = dev(f.a_mk[:M].reshape(-1))
            dC = torch.zeros(M * NC, dtype=torch.int16, device="cuda")
            dR = torch.from_numpy(rows).cuda()
            desc = B.GroupedGemmDesc(M, f.N, f.K, f.G, B.Layout(W.row_major_spec(M, f.K)), useL, B.Layout(W.row_major_spec(M, NC)),
                                     M * f.K, f.b_gnk.size, M * NC, in_dtype=dt, out_dtype=dt,
                                     epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE)
            wall, devms = time_loop(lambda i: B.axe_gemm_grouped(desc, dA, dBuse, dC, dR), steps, warmup)
            active = int((np.diff(rows) > 0).sum())
            nbytes = 2.0 * (active * f.N * f.K + M * f.K + M * NC)
            which = B.axe_gemm_grouped_kernel(desc)
            kernel = {B.AXE_GROUPED_STREAM: "streaming (split K)", B.AXE_GROUPED_TILES_128: "tiles of 128 x 256"}.get(which, "tiles of 256 x 256")
            r = {"M": M, "active_experts": active, "kernel": kernel, "kernel_ms": devms, "algorithmic_bytes": nbytes,
                 "GBps": nbytes / (devms * 1e-3) / 1e9, "tflops": 2.0 * M * f.N * f.K / (devms * 1e-3) / 1e12}
            r["frac_of_hbm_peak"] = r["GBps"] / PEAK["hbm"]
            out["sweep"].setdefault(str(tokens), {})[name] = r
            layer[tokens] += devms
            log(f"[bench] MoE {name}{' + gated activation' if gated else ''} {dtype}, {tokens} tokens (M={M}, {active} experts with rows, {kernel}): "
                f"{devms*1e3:.1f} us, {r['GBps']:.0f} GB/s ({100*r['frac_of_hbm_peak']:.0f}% of HBM peak), {r['tflops']:.0f} TFLOP/s")
            if tokens == top:                            # without the epilogue, plain against blocked weights
                dCw = torch.zeros(M * f.N, dtype=torch.int16, device="cuda")
                for label, lay, buf in (("plain", plainL, dB), ("blocked", blkL, dBblk)):
                    d2 = B.GroupedGemmDesc(M, f.N, f.K, f.G, B.Layout(W.row_major_spec(M, f.K)), lay, B.Layout(W.row_major_spec(M, f.N)),
                                           M * f.K, f.b_gnk.size, M * f.N, in_dtype=dt, out_dtype=dt)
                    wall, d_ms = time_loop(lambda i: B.axe_gemm_grouped(d2, dA, buf, dCw, dR), steps, warmup)
                    r[label + "_weights_no_epilogue_ms"] = d_ms
                log(f"[bench]   {name} at {tokens} tokens without epilogue: plain weights {r['plain_weights_no_epilogue_ms']*1e3:.0f} us, "
                    f"blocked weights {r['blocked_weights_no_epilogue_ms']*1e3:.0f} us")
                del dCw
            del dA, dC
        packed[name] = (dBuse, useL)
        del dB, dBblk, dBuse
    for tokens in sweep:
        out["sweep"][str(tokens)]["layer_kernel_ms"] = layer[tokens]
    log("[bench] MoE layer expert compute (gemm1 + activation, gemm2), us by tokens: " +
        ", ".join(f"{t}: {layer[t]*1e3:.0f}" for t in sweep))
    # both GEMMs as one launch (axe_gemm_grouped_pair: gemm2's row blocks start when gemm1's tiles for those rows are
    # stored), where the library shares the launch; the two-launch time through the same entry point beside it
    f1, f2 = full["gemm1"], full["gemm2"]
    fused = {}
    for tokens in sweep:
        rows = W.moe_group_rows(tokens, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
        M, I = int(rows[-1]), f1.N // 2
        d1 = B.GroupedGemmDesc(M, f1.N, f1.K, f1.G, B.Layout(W.row_major_spec(M, f1.K)), packed["gemm1"][1], B.Layout(W.row_major_spec(M, I)),
                               M * f1.K, f1.b_gnk.size, M * I, in_dtype=dt, out_dtype=dt, epilogue=B.AXE_EPI_SWIGLU)
        d2 = B.GroupedGemmDesc(M, f2.N, f2.K, f2.G, B.Layout(W.row_major_spec(M, f2.K)), packed["gemm2"][1], B.Layout(W.row_major_spec(M, f2.N)),
                               M * f2.K, f2.b_gnk.size, M * f2.N, in_dtype=dt, out_dtype=dt)
        if not B.axe_gemm_grouped_pair_fused(d1, d2):
            continue
        dA = dev(f1.a_mk[:M].reshape(-1))
        dH = torch.zeros(M * I, dtype=torch.int16, device="cuda")
        dC = torch.zeros(M * f2.N, dtype=torch.int16, device="cuda")
        dR = torch.from_numpy(rows).cuda()
        sync = torch.zeros(M + 1, dtype=torch.int32, device="cuda")
        _, two = time_loop(lambda i: B.axe_gemm_grouped_pair(d1, d2, dA, packed["gemm1"][0], dH, packed["gemm2"][0], dC, dR, None), steps, warmup)
        _, one = time_loop(lambda i: B.axe_gemm_grouped_pair(d1, d2, dA, packed["gemm1"][0], dH, packed["gemm2"][0], dC, dR, sync), steps, warmup)
        B.axe_gemm_grouped_pair_status(sync, M)
        out["sweep"][str(tokens)]["layer_two_launches_ms"] = two
        out["sweep"][str(tokens)]["layer_one_launch_ms"] = one
        fused[tokens] = (two, one)
        del dA, dH, dC
    if fused:
        log("[bench] MoE layer as one launch with tile-level hand-over (two launches -> one), us by tokens: " +
            ", ".join(f"{t}: {a*1e3:.0f} -> {b*1e3:.0f}" for t, (a, b) in fused.items()))
    return out


def bench_grouped_fp8(steps, warmup, sweep=(1, 8, 64, 256, 512, 2048, 4096)):
    """The same layer with e4m3 weights and activations: E8M0 block scales (one per row and 128-wide k block
    for the activations, one per 128 x 128 block for the weights), bf16 output; gemm1 with the gated activation.  The
    weights are half the bytes of the fp16 layer; bound: HBM.  Kernels chosen by the library: the weight-streaming
    kernel at decode sizes, the tile kernel on the matrix cores' scale path from 9 - 16 rows per expert on."""
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    top = max(sweep)
    out = {"dtype": "fp8 e4m3, E8M0 scales", "sweep": {}}
    layer = {t: 0.0 for t in sweep}
    rows_top = W.moe_group_rows(top, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
    for name, N, K in (("gemm1", 2 * W.MOE_INTER, W.MOE_HIDDEN), ("gemm2", W.MOE_HIDDEN, W.MOE_INTER)):
        gated = name == "gemm1"
        NC = N // 2 if gated else N
        f = W.gemm_grouped_fp8(rows_top, N, K, W.SEED_BASE + 21 + gated, scale_dtype="e8m0")
        plainL = B.Layout(W.grouped_gemm_specs(f)[1])
        useL = B.Layout(W.gated_b_spec(K, N, f.G)) if gated else plainL
        dB = dev(f.b_gnk.reshape(-1))
        if gated:                                        # gate and up rows interleaved: packed by axe_relayout (untimed)
            dBp = torch.empty_like(dB)
            B.axe_relayout(plainL, useL, (f.G, K, N), dB, dBp)
            dB = dBp
        sb = torch.from_numpy(f.scale_b).cuda()
        for tokens in sweep:
            rows = W.moe_group_rows(tokens, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
            M = int(rows[-1])
            dA, sa = dev(f.a_mk[:M].reshape(-1)), torch.from_numpy(f.scale_a[:M]).cuda()
            dC = torch.zeros(M * NC, dtype=torch.int16, device="cuda")
            dR = torch.from_numpy(rows).cuda()
            desc = B.GroupedGemmDesc(M, N, K, f.G, B.Layout(W.row_major_spec(M, K)), useL, B.Layout(W.row_major_spec(M, NC)),
                                     M * K, f.b_gnk.size, M * NC, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16,
                                     epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, scale_a=sa, scale_b=sb,
                                     scale_dtype=B.AXE_SCALE_E8M0)
            wall, devms = time_loop(lambda i: B.axe_gemm_grouped(desc, dA, dB, dC, dR), steps, warmup)
            active = int((np.diff(rows) > 0).sum())
            nbytes = active * N * K + M * K + 2.0 * M * NC
            kernel = {B.AXE_GROUPED_STREAM: "streaming", B.AXE_GROUPED_TILES_128: "tiles of 128 x 256"}.get(B.axe_gemm_grouped_kernel(desc), "tiles of 256 x 256")
            r = {"M": M, "active_experts": active, "kernel": kernel, "kernel_ms": devms, "algorithmic_bytes": nbytes,
                 "GBps": nbytes / (devms * 1e-3) / 1e9, "tflops": 2.0 * M * N * K / (devms * 1e-3) / 1e12}
            r["frac_of_hbm_peak"] = r["GBps"] / PEAK["hbm"]
            out["sweep"].setdefault(str(tokens), {})[name] = r
            layer[tokens] += devms
            log(f"[bench] MoE {name}{' + gated activation' if gated else ''} fp8, {tokens} tokens (M={M}, {active} experts with rows, {kernel}): "
                f"{devms*1e3:.1f} us, {r['GBps']:.0f} GB/s ({100*r['frac_of_hbm_peak']:.0f}% of HBM peak), {r['tflops']:.0f} TFLOP/s")
            del dA, dC
        del dB
    for tokens in sweep:
        out["sweep"][str(tokens)]["layer_kernel_ms"] = layer[tokens]
    log("[bench] MoE layer expert compute in fp8, us by tokens: " + ", ".join(f"{t}: {layer[t]*1e3:.0f}" for t in sweep))
    return out


def bench_eval(steps, warmup):
    import torch
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    rows = cols = 8192
    L = B.Layout(W.blocked_swizzled_spec(rows, cols))
    n = rows * cols
    outs = [torch.empty((n, 1, 1), dtype=torch.int64, device="cuda") for _ in range(2)]      # 512 MiB each: nothing stays in a cache
    wall, devms = time_loop(lambda i: B.axe_layout_eval(L, (rows, cols), n, None, outs[i % 2]), steps, warmup)
    r = {"points": n, "kernel_ms": devms, "Gpoints_per_s": n / (devms * 1e-3) / 1e9, "GBps_written": n * 8 / (devms * 1e-3) / 1e9}
    r["frac_of_hbm_peak"] = r["GBps_written"] / PEAK["hbm"]
    log(f"[bench] layout eval 2^26 points: {devms:.4f} ms, {r['Gpoints_per_s']:.1f} Gpoint/s, {r['GBps_written']:.0f} GB/s written "
        f"({100 * r['frac_of_hbm_peak']:.1f}% of HBM peak)")
    return r


def bench_ceilings(g3, g5, steps=20, warmup=5):
    """Measured ceilings for context: register-only MFMA loops (the instruction, wave count and
    accumulator walk of the two 256 x 256 kernels) on a sample of the real operands, and a plain
    device-to-device copy of the relayout's size."""
    import ctypes as C
    import torch
    from paper_2601_19092_amd import binding as B
    path = os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_probe.so")
    if not os.path.exists(path):
        sys.exit(f"bench.py: {path} is missing (run __graft_entry__.build())")
    P = C.CDLL(path)
    P.axe_probe_mfma.restype = C.c_int
    P.axe_probe_mfma.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_size_t,
                                 C.POINTER(C.c_double), C.c_void_p]
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(cus * 512, dtype=torch.float32, device="cuda")
    out = {}
    for key, g, fp8, nbytes, iters in (("mfma_bf16", g3, 0, 16 * 256 * 16, 8000), ("mfma_fp8", g5, 1, 12 * 256 * 32, 4000)):
        # rows from the middle of A: 64 or 96 KiB of consecutive operand codes
        sample = dev(g.a_mk.reshape(-1).view(np.uint8)[g.a_mk.nbytes // 2:][:nbytes].copy())
        flops = C.c_double(0.0)
        def launch(i):
            rc = P.axe_probe_mfma(fp8, sample.data_ptr(), nbytes, iters, sink.data_ptr(), sink.numel(), C.byref(flops),
                                  torch.cuda.current_stream().cuda_stream)
            if rc:
                sys.exit(f"bench.py: axe_probe_mfma failed ({rc})")
        _, devms = time_loop(launch, steps, warmup)
        out[key + "_register_only_tflops"] = flops.value / (devms * 1e-3) / 1e12
    # the same bf16 loop with its MFMAs issued in other orders: what the order alone does to the sustained rate
    P.axe_probe_mfma_walk.restype = C.c_int
    P.axe_probe_mfma_walk.argtypes = P.axe_probe_mfma.argtypes
    sample = dev(g3.a_mk.reshape(-1).view(np.uint8)[g3.a_mk.nbytes // 2:][:16 * 256 * 16].copy())
    walks = {"kernel (row pairs, alternating direction)": 0, "row by row": 1, "row pairs, one direction": 2,
             "diagonal": 3, "rows in fours": 4}
    by_walk = {k: [] for k in walks}
    for rnd in range(2):                                            # alternating, so that drift of the clock hits all alike
        for name, walk in walks.items():
            flops = C.c_double(0.0)
            def launch(i, walk=walk):
                rc = P.axe_probe_mfma_walk(walk, sample.data_ptr(), sample.numel(), 4000, sink.data_ptr(), sink.numel(), C.byref(flops),
                                           torch.cuda.current_stream().cuda_stream)
                if rc:
                    sys.exit(f"bench.py: axe_probe_mfma_walk failed ({rc})")
            _, devms = time_loop(launch, 20, 5)
            by_walk[name].append(flops.value / (devms * 1e-3) / 1e12)
    out["mfma_bf16_register_only_tflops_by_walk"] = {k: sum(v) / len(v) for k, v in by_walk.items()}
    log("[bench] register-only bf16 MFMA loop by order of the 64 MFMAs of a pass: " +
        ", ".join(f"{k} {v:.0f}" for k, v in out["mfma_bf16_register_only_tflops_by_walk"].items()) + " TFLOP/s")
    n = 8192 * 8192
    pairs = [(torch.randint(-30000, 30000, (n,), dtype=torch.int16, device="cuda"),
              torch.empty(n, dtype=torch.int16, device="cuda")) for _ in range(4)]
    _, devms = time_loop(lambda i: pairs[i % 4][1].copy_(pairs[i % 4][0]), 40, 10)
    out["device_copy_GBps"] = 2.0 * n * 2 / (devms * 1e-3) / 1e9
    # plain HBM streams with the relayout's access shape (128-bit non-temporal, four per thread), same size, same rotation
    P.axe_probe_stream.restype = C.c_int
    P.axe_probe_stream.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    for key, kind, moved in (("stream_copy_GBps", 0, 2.0), ("stream_read_GBps", 1, 1.0), ("stream_write_GBps", 2, 1.0)):
        def launch(i, kind=kind):
            rc = P.axe_probe_stream(kind, pairs[i % 4][0].data_ptr(), pairs[i % 4][1].data_ptr(), n * 2, torch.cuda.current_stream().cuda_stream)
            if rc:
                sys.exit(f"bench.py: axe_probe_stream failed ({rc})")
        _, devms = time_loop(launch, 40, 10)
        out[key] = moved * n * 2 / (devms * 1e-3) / 1e9
    log(f"[bench] measured ceilings: register-only MFMA loop bf16 {out['mfma_bf16_register_only_tflops']:.0f} TFLOP/s, "
        f"fp8 {out['mfma_fp8_register_only_tflops']:.0f} TFLOP/s on samples of the inputs; "
        f"128 MiB rotating over 4 pairs: library device copy {out['device_copy_GBps']:.0f} GB/s, plain 128-bit non-temporal "
        f"stream copy {out['stream_copy_GBps']:.0f} GB/s (read + write), read only {out['stream_read_GBps']:.0f} GB/s, "
        f"write only {out['stream_write_GBps']:.0f} GB/s")
    return out


def cpu_baseline(g, budget_rows=2048):
    """The CPU oracle as it stands, on the first `budget_rows` rows of the same GEMM (all rows when budget_rows is
    None), and the oracle's relayout of the whole of configuration 2 beside it."""
    from oracle import axe_ref as R
    from oracle.axe_layout import Layout
    from paper_2601_19092_amd import workloads as W
    rows = None if budget_rows is None or budget_rows >= g.M else np.arange(budget_rows)
    nrows = g.M if rows is None else budget_rows
    R.gemm_ref(g.a_mk[:2], g.b_nk.T[:, :2], R.AXE_BF16)        # builds / loads the C oracle outside the timing
    t0 = time.perf_counter()
    R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_BF16, rows=rows)
    dt = time.perf_counter() - t0
    fl = 2.0 * nrows * g.N * g.K
    # relayout oracle (NumPy scatter through both layouts' evaluations), whole configuration 2
    n = 8192
    words = W.config2("uniform").reshape(-1)
    dst = np.zeros(n * n, dtype=np.uint16)
    t1 = time.perf_counter()
    R.relayout_ref(Layout.from_spec(W.row_major_spec(n, n)), Layout.from_spec(W.blocked_swizzled_spec(n, n)), (n, n), words, dst)
    dt_r = time.perf_counter() - t1
    what = f"all {g.M} rows" if rows is None else f"rows 0..{budget_rows - 1}"
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": R.oracle_threads(), "kind": "oracle",
            "sample": f"{what} of C (all {g.N} columns, K = {g.K}) of the same bf16 GEMM, plain fp64 triple loop, {dt:.1f} s",
            "whole_config": rows is None,
            "relayout_cfg2": {"value": 2.0 * n * n * 2 / dt_r / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                              "sample": f"the whole 8192 x 8192 bf16 relayout of configuration 2 (NumPy evaluation of both layouts + scatter), {dt_r:.1f} s"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--only", default="", help="comma list of: gemm,relayout,fp8,shard,ragged,grouped,small,eval,ceilings,cpu (default all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cpu-full", action="store_true", help="time the CPU oracle on the whole of configuration 3 (about 1.5 minutes on 16 cores) instead of a quarter of its rows")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding across GPUs); use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2601_19092_amd import binding as B
    from paper_2601_19092_amd import workloads as W
    B.lib()                                                  # fails loudly if the HIP library is missing
    only = set(filter(None, args.only.split(",")))
    want = lambda k: not only or k in only

    log("[bench] generating configuration 3 (bf16 GEMM 8192^3) on the host ...")
    g3 = W.config3()
    head, _ = bench_gemm("bf16 GEMM M=N=K=8192, A row-major, B column-major, bf16 out", g3, args.steps, args.warmup,
                         min_warm_ms=0, headline=True)   # clocks settled first, then exactly args.warmup untimed steps
    comp = {}
    if want("relayout"):
        comp["relayout_cfg2"] = bench_relayout(max(20, args.steps), args.warmup)
        comp["relayout_transpose_8192"] = bench_transpose(max(20, args.steps), args.warmup)
    if want("shard"):
        comp["gemm_cfg4_tp_shard"], _ = bench_gemm("bf16 GEMM M=4096 K=8192 N=3584 (1 of 8 shards)", W.config4(),
                                                   args.steps, args.warmup, device_axis=True)
    if want("ragged"):
        comp["gemm_ragged_4000"], _ = bench_gemm("bf16 GEMM M=N=4000 K=4096 (edges that do not fill a 256x256 tile)",
                                                 W.gemm_bf16(4000, 4000, 4096, W.SEED_BASE + 7, std_b=4096 ** -0.5),
                                                 args.steps, args.warmup)
    g5 = W.config5() if (want("fp8") or want("ceilings")) else None
    if want("fp8"):
        comp["gemm_cfg5_fp8_block_scaled"], _ = bench_gemm("fp8 e4m3 GEMM 8192^3, fp32 128x128 block scales", g5,
                                                           max(10, args.steps // 2), args.warmup)
    if want("fp8"):
        comp["gemm_fp8_e8m0_block_scaled"], _ = bench_gemm(
            "fp8 e4m3 GEMM 8192^3, E8M0 (power-of-two) 128x128 block scales on the MFMA scale path",
            W.gemm_fp8(8192, 8192, 8192, W.SEED_BASE + 5, scaled="e8m0"), max(10, args.steps // 2), args.warmup)
    if want("fp8"):
        # activations scaled per row and 128-wide k block (one E8M0 code each), weights per 128 x 128 block
        gr = W.gemm_fp8(8192, 8192, 8192, W.SEED_BASE + 6, scaled="e8m0")
        gr.scale_a = np.random.default_rng(W.SEED_BASE + 6).integers(124, 131, (8192, 64)).astype(np.uint8)
        comp["gemm_fp8_e8m0_row_scaled"], _ = bench_gemm(
            "fp8 e4m3 GEMM 8192^3, E8M0 scales: one per row and k block of A, one per 128x128 block of B, on the MFMA scale path",
            gr, max(10, args.steps // 2), args.warmup, scale_a_rows=1)
    if want("grouped"):
        comp["moe_grouped_gemm"] = bench_grouped(max(10, args.steps // 3), args.warmup)
        comp["moe_grouped_gemm_fp8"] = bench_grouped_fp8(max(10, args.steps // 3), args.warmup)
    if want("small"):
        comp["gemm_cfg1_256"], _ = bench_gemm("bf16 GEMM 256^3, fp32 out, 64x64x32 tiles", W.config1(),
                                              max(200, args.steps), max(200, args.warmup), n_sets=1)
        step1, _sets1, _ = gemm_setup(W.config1(), 1)
        comp["gemm_cfg1_256"]["graph_replay_us_per_launch"] = graph_replay_us(step1)
        log(f"[bench] bf16 GEMM 256^3 recorded 64 times into a HIP graph and replayed: "
            f"{comp['gemm_cfg1_256']['graph_replay_us_per_launch']:.2f} us per launch")
    if want("eval"):
        comp["layout_eval"] = bench_eval(20, 5)
    if want("ceilings"):
        c = bench_ceilings(g3, g5)
        c["gemm_cfg3_frac_of_measured"] = head["kernel_tflops"] / c["mfma_bf16_register_only_tflops"]
        if "gemm_cfg5_fp8_block_scaled" in comp:
            c["gemm_cfg5_frac_of_measured"] = comp["gemm_cfg5_fp8_block_scaled"]["kernel_tflops"] / c["mfma_fp8_register_only_tflops"]
        if "relayout_cfg2" in comp:
            c["relayout_cfg2_frac_of_measured"] = comp["relayout_cfg2"]["rotating"]["GBps"] / c["device_copy_GBps"]
            c["relayout_cfg2_frac_of_stream_copy"] = comp["relayout_cfg2"]["rotating"]["GBps"] / c["stream_copy_GBps"]
        comp["measured_ceilings"] = c
    cpu = None
    if not args.no_cpu and want("cpu"):
        log("[bench] timing the CPU oracle on a bounded sample ...")
        cpu = cpu_baseline(g3, None if args.cpu_full else 2048)
        log(f"[bench] cpu oracle: {cpu['value'] * 1e3:.2f} GFLOP/s on {cpu['cores']} threads")

    flops = 2.0 * g3.M * g3.N * g3.K
    line = {
        "metric": "GEMM TFLOP/s + % MFMA peak; relayout GB/s + % HBM peak (1 GPU)",
        "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 3: bf16 GEMM M=N=K=8192, A row-major, B column-major, N(0, K^-1/2) inputs, "
                               "fp32 accumulate, bf16 output; 256x256x64 tiles described as Axe layouts"},
        "roofline": {"bound": "mfma", "achieved": head["kernel_tflops"], "peak": PEAK["bf16"], "unit": "TFLOP/s",
                     "frac": head["kernel_tflops"] / PEAK["bf16"], "traffic": None,
                     "kernel": "gemm_bf16_256_kernel", "flops_per_launch": flops, "kernel_ms": head["kernel_ms"],
                     "per_launch_kernel_ms": head["per_launch_kernel_ms"]},
        "clock_settle": head["settle"],           # extra untimed launches before the --warmup steps (see settle())
        "cpu_baseline": cpu,
        "companions": comp,
    }
    tr = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tr):
        try:
            line["roofline"]["traffic"] = json.load(open(tr)).get("gemm_bf16_256_kernel_bytes_per_launch")
        except Exception:
            pass
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
