#!/usr/bin/env python3
"""Benchmark of the MI355X linear-attention hot path.

One "step" is one forward pass of the attention core of one layer over all
heads of the workload: state reduction + fixed-order reduce + apply
(bidirectional workloads), i.e. every token of Q, K, V read once and O written
once.  Inputs are synthetic (i.i.d. Gaussian times 0.5, bf16), generated on the
device and resident in HBM before the timed region starts; buffer sets rotate
so that repeats are not served from the 256 MB Infinity Cache.

Prints ONE JSON line.  `value` is tokens/s of the layer (B*N / time per step) on
the headline workload: the 720p-like bidirectional layer (B = 2, 64 heads of
75 600 tokens), the largest configuration of the method that one call covers.
`roofline` refers to the slower of the two kernels of a step (state or apply),
timed with HIP events on the launch stream over a second pass of the same steps
(events between kernels cost a few microseconds, so they stay out of `value`).
`cpu_baseline` is the float64 oracle timed on the host cores on the same
workload.  The 480p-like layer is reported under `secondary`, the block-causal
workloads under `block_stream` (with the latency and the device memory of every
block), the paper's head geometry under `geometry_h20d112`.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix rate, published

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "traffic_table.txt")


def measured_traffic():
    """HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this file, read from
    profiles/traffic_table.txt: one line per (kernel, workload) with the two counters in KiB per dispatch, the
    factors that scale them to bytes moved (what the same counters read for a plain device copy of known
    size) and the fingerprint of the kernel sources the run was made on.  Returns
    {(kernel, workload): (bytes, fingerprint)}."""
    table = {}
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                parts = line.split()
                if len(parts) != 7 or line.lstrip().startswith("#"):
                    continue
                kernel, workload, fetch, write, fs, wsc, fp = parts
                table[(kernel, workload)] = (int((float(fetch) * float(fs) + float(write) * float(wsc)) * 1024), fp)
    except OSError:
        pass
    return table


def traffic_of(table, kernel, workload, fingerprint):
    """(bytes or None, note): counters taken on other kernel sources than the ones now built say nothing."""
    if (kernel, workload) not in table:
        return None, "no counter run kept for this kernel and workload"
    nbytes, fp = table[(kernel, workload)]
    if fp != fingerprint:
        return None, f"counter run was made on kernel sources {fp}, this build is {fingerprint}"
    return nbytes, "profiles/traffic_table.txt"


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bidir_720p", choices=["bidir_480p", "bidir_720p", "bidir_480p_h20d112"])
    ap.add_argument("--no-secondary", action="store_true", help="skip the 480p-like bidirectional layer")
    ap.add_argument("--no-apply-variants", action="store_true",
                    help="skip the A/B timings of the apply kernel's measurement variants")
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough for > 1.5 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-block-stream", action="store_true")
    ap.add_argument("--no-rope", action="store_true", help="skip the RoPE-variant timings")
    ap.add_argument("--no-tconv", action="store_true", help="skip the Mix-FFN temporal-convolution timings")
    ap.add_argument("--no-d112", action="store_true",
                    help="skip the timings in the geometry of the paper's 2B model (20 heads of 112 features)")
    ap.add_argument("--stream-blocks", type=int, default=80)
    ap.add_argument("--no-stream-ceiling", action="store_true",
                    help="skip the pure read / pure copy yardsticks")
    ap.add_argument("--calibration-copy", type=int, default=0,
                    help="also run this many plain device copies of one token tensor (known size: "
                         "the same bytes read and written), for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE")
    return ap.parse_args()


def _randn_bf16(shape, gen):
    import torch
    return (torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen) * 0.5).to(torch.bfloat16)


def _rope_table(w, torch, t0=0):
    """Full rotation table [N][d/2][2] of the workload's token grid (device tensor)."""
    import sv_workloads as wl
    return torch.from_numpy(wl.rope_table_3d(*w.grid, w.d, t0=t0)).cuda()


def _rope_3d(w, torch, sv, t0=0):
    """The same embedding as three per-axis tables (sv.Rope3D)."""
    import sv_workloads as wl
    return sv.Rope3D.from_tensors(*(torch.from_numpy(t).cuda()
                                    for t in wl.rope_tables_3d_factored(*w.grid, w.d, t0=t0)))


def _is_3d(rope):
    return rope is not None and rope.__class__.__name__ == "Rope3D"


def bench_bidirectional(w, steps, warmup, n_sets, sv, torch, rope=None, sets=None):
    """`rope`: a device table or an sv.Rope3D -> the _rope / _rope3d entry points are timed instead of
    the plain ones."""
    B, H, N, d = w.B, w.H, w.N, w.d
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    if n_sets <= 0:
        n_sets = max(2, -(-int(1.5e9) // w.algorithmic_bytes))
    if sets is None:
        sets = []
        for _ in range(n_sets):
            q, k, v = (_randn_bf16((B, H, N, d), gen) for _ in range(3))
            sets.append((q, k, v, torch.empty_like(q)))
    n_sets = len(sets)
    S = torch.empty((B, H, d, d), dtype=torch.float32, device="cuda")
    z = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = torch.empty(sv.sv_linattn_workspace_bytes(B, H, N, d), dtype=torch.uint8, device="cuda")
    dsc = sv.desc_of(sets[0][0])
    stream = torch.cuda.current_stream()

    def step(i, ev=None):
        q, k, v, o = sets[i % n_sets]
        if ev:
            ev[0].record(stream)
        if rope is None:
            sv.sv_linattn_state(k, v, dsc, 0, N, 0, S, z, ws, stream=stream)
        elif _is_3d(rope):
            sv.sv_linattn_state_rope3d(k, v, dsc, rope, 0, N, 0, S, z, ws, stream=stream)
        else:
            sv.sv_linattn_state_rope(k, v, dsc, rope, 0, N, 0, S, z, ws, stream=stream)
        if ev:
            ev[1].record(stream)
        if rope is None:
            sv.sv_linattn_apply(q, dsc, 0, N, S, z, w.eps, o, stream=stream)
        elif _is_3d(rope):
            sv.sv_linattn_apply_rope3d(q, dsc, rope, 0, N, S, z, w.eps, o, stream=stream)
        else:
            sv.sv_linattn_apply_rope(q, dsc, rope, 0, N, S, z, w.eps, o, stream=stream)
        if ev:
            ev[2].record(stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps, nothing else on the stream
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # second pass of `steps` steps with HIP events on the launch stream around each call: per-kernel
    # durations (an event between two kernels costs a few microseconds, so this pass is not `value`)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(steps):
        step(i, events[i])
    torch.cuda.synchronize()
    wall_ev = time.perf_counter() - t1
    t_state = [e[0].elapsed_time(e[1]) for e in events]      # ms
    t_apply = [e[1].elapsed_time(e[2]) for e in events]
    if sv.sv_linattn_workspace_status(ws, B, H, d) != 0:
        raise RuntimeError("an in-kernel wait timed out during the benchmark: its figures mean nothing")
    return {
        "ms_per_step": wall / steps * 1e3, "ms_per_step_with_events": wall_ev / steps * 1e3,
        "ms_state": statistics.mean(t_state), "ms_apply": statistics.mean(t_apply),
        "n_sets": n_sets, "sets": sets,
    }


def bench_block_stream(w, n_blocks, sv, torch, rope=False, ceiling=False, traffic=None):
    """Whole stream enqueued back to back, one event pair per block; no host sync inside.
    `rope`: False, "table" (sv_block_linattn_step_rope, one full table per block) or "3d"
    (sv_block_linattn_step_rope3d, per-axis tables; the frame table of each block continues the
    time axis)."""
    B, H, N, d = w.B, w.H, w.N, w.d
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    blocks = []
    for _ in range(n_blocks):
        q, k, v = (_randn_bf16((B, H, N, d), gen) for _ in range(3))
        blocks.append((q, k, v, torch.empty_like(q)))
    S = torch.zeros((B, H, d, d), dtype=torch.float32, device="cuda")
    z = torch.zeros((B, H, d), dtype=torch.float32, device="cuda")
    ws = torch.empty(sv.sv_linattn_workspace_bytes(B, H, N, d), dtype=torch.uint8, device="cuda")
    lib_bytes = S.numel() * 4 + z.numel() * 4 + ws.numel()
    dsc = sv.desc_of(blocks[0][0])
    stream = torch.cuda.current_stream()
    if rope == "3d":
        tables = [_rope_3d(w, torch, sv, t0=m * w.grid[0]) for m in range(n_blocks)]
    elif rope:
        tables = [_rope_table(w, torch, t0=m * w.grid[0]) for m in range(n_blocks)]
    else:
        tables = None
    step_rope = sv.sv_block_linattn_step_rope3d if rope == "3d" else sv.sv_block_linattn_step_rope

    def one(m):
        q, k, v, o = blocks[m]
        if tables is None:
            sv.sv_block_linattn_step(q, k, v, dsc, S, z, w.eps, o, ws, stream=stream)
        else:
            step_rope(q, k, v, dsc, tables[m], S, z, w.eps, o, ws, stream=stream)

    def run(events=None):
        S.zero_()
        z.zero_()
        for m in range(n_blocks):
            if events:
                events[m][0].record(stream)
            one(m)
            if events:
                events[m][1].record(stream)

    run()                                           # warm-up pass over the stream
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    mem_before = torch.cuda.memory_allocated()
    # pass 1: one event pair around the whole stream (throughput); a short stream lasts well under a
    # millisecond, so one hiccup of the enqueueing host thread would dominate it: best of three.  An untimed
    # pass of the same stream is enqueued right in front of the timed one, with no host sync between them: the
    # first kernels after an idle spell run slower (a block_480p step takes 34 us then, 25 after), and a layer of a
    # model never starts on an idle device.
    stream_ms = float("inf")
    for _ in range(3):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        run()
        S.zero_()
        z.zero_()
        a.record(stream)
        for m in range(n_blocks):
            one(m)
        b.record(stream)
        torch.cuda.synchronize()
        stream_ms = min(stream_ms, a.elapsed_time(b))
    # pass 2: per-block latency, one event pair per block.  The stream is run three times and each block's figure
    # is the median of its three (a lone stall of the device - a refresh, a clock step - otherwise decides `max`);
    # the spread of the three passes is reported beside it.
    passes = []
    for _ in range(3):
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in blocks]
        run(events)
        torch.cuda.synchronize()
        passes.append([e[0].elapsed_time(e[1]) * 1e3 for e in events])            # us
    lat = [statistics.median(p[m] for p in passes) for m in range(n_blocks)]
    lat_worst = [max(p[m] for p in passes) for m in range(n_blocks)]
    peak_extra = torch.cuda.max_memory_allocated() - mem_before
    # pass 2b: device memory after every block (the block is waited for, so this pass is not timed): bytes
    # this process holds through the allocator, and bytes in use on the whole device
    mem_alloc, mem_device = [], []
    S.zero_()
    z.zero_()
    for m in range(n_blocks):
        one(m)
        torch.cuda.synchronize()
        free_b, total_b = torch.cuda.mem_get_info()
        mem_alloc.append(int(torch.cuda.memory_allocated()))
        mem_device.append(int(total_b - free_b))
    if sv.sv_linattn_workspace_status(ws, B, H, d) != 0:
        raise RuntimeError("an in-kernel wait timed out during the block stream: its figures mean nothing")
    # pass 3: the whole stream recorded once into a HIP graph and replayed (the workspace is switched
    # to device-side epochs for that)
    sv.sv_linattn_workspace_init(ws, B, H, d, stream=stream)
    run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cap = torch.cuda.current_stream()
        for m in range(n_blocks):
            q, k, v, o = blocks[m]
            if tables is None:
                sv.sv_block_linattn_step(q, k, v, dsc, S, z, w.eps, o, ws, stream=cap)
            else:
                step_rope(q, k, v, dsc, tables[m], S, z, w.eps, o, ws, stream=cap)
    graph.replay()
    torch.cuda.synchronize()
    ga, gb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    graph.replay()                                  # untimed, right in front of the timed replays (see pass 1)
    ga.record(stream)
    for _ in range(reps):
        graph.replay()
    gb.record(stream)
    torch.cuda.synchronize()
    graph_us = ga.elapsed_time(gb) * 1e3 / (reps * n_blocks)
    tail = lat[1:] if len(lat) > 1 else lat
    med = statistics.median(tail)
    xs = list(range(len(tail)))
    mx, my = statistics.mean(xs), statistics.mean(tail)
    slope = (sum((x - mx) * (y - my) for x, y in zip(xs, tail)) / max(1e-30, sum((x - mx) ** 2 for x in xs))
             if len(tail) > 1 else 0.0)
    per_block_us = stream_ms * 1e3 / n_blocks
    out = {
        "workload": w.name, "rope": ("table" if rope is True else rope), "blocks": n_blocks, "tokens_per_block": N,
        "us_per_block_stream": per_block_us, "us_per_block_graph_replay": graph_us,
        "tokens_per_s": B * N / (per_block_us * 1e-6),
        "hbm_GBps": w.algorithmic_bytes / (per_block_us * 1e-6) / 1e9,
        "hbm_frac": w.algorithmic_bytes / (per_block_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
        "latency_us": {"first": lat[0], "min": min(tail), "median": med, "max": max(tail),
                       "max_over_median": max(tail) / med, "slope_us_per_block": slope},
        "latency_us_per_block": [round(x, 2) for x in lat],
        "latency_us_per_block_worst_of_3_passes": [round(x, 2) for x in lat_worst],
        "library_bytes": lib_bytes, "peak_new_device_bytes_during_stream": int(peak_extra),
        # after every block: bytes held through the allocator and bytes in use on the device (inputs and
        # outputs of all blocks are resident from the start; the library itself holds library_bytes throughout)
        "allocated_bytes_after_block": mem_alloc, "device_bytes_in_use_after_block": mem_device,
        "memory_constant_over_stream": len(set(mem_alloc)) == 1,
    }
    if traffic is not None:
        nbytes, note = traffic
        gbps = w.algorithmic_bytes / (per_block_us * 1e-6) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "block_step_mfma", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                           "frac": gbps / HBM_PEAK_GBPS, "traffic": nbytes, "traffic_source": note,
                           "algorithmic_bytes_per_launch": w.algorithmic_bytes, "avg_launch_ms": per_block_us * 1e-3}
    if ceiling:
        # what the device gives two dependent passes that only move the block's bytes: a pure read of K_b, V_b,
        # then a pure copy of Q_b's size into O_b's (kernels of include/sv_measure.h, timed like the blocks)
        c = bench_stream_ceiling(w.algorithmic_bytes // 2, sv, torch)
        floor_us = c["read"]["us"] + c["copy"]["us"]
        out["stream_ceiling"] = {"read_us": c["read"]["us"], "copy_us": c["copy"]["us"], "bytes_each": c["read"]["bytes"],
                                 "read_then_copy_us": floor_us}
        out["frac_of_stream_ceiling"] = floor_us / per_block_us
    return out


def bench_stream_ceiling(nbytes, sv, torch, reps=12):
    """What the device gives kernels that only move bytes (include/sv_measure.h): a pure read of
    `nbytes` and a pure copy that reads nbytes/2 and writes nbytes/2 (the traffic of one state and
    of one apply launch), best average over a few launch shapes, buffers rotated so that the last
    level cache cannot serve repeats.  Context for `roofline`, which is quoted against the published peak."""
    n_sets = max(2, -(-int(1.5e9) // nbytes))
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(n_sets)]
    for i, b in enumerate(bufs):
        b.fill_(i + 1)
    half = nbytes // 2 // 16 * 16
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    out = {}
    for kind in ("read", "copy"):
        best = None
        for wgs in (1024, 4096, 8192, 16384, 65536):
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps + 2)]
            for i, (e0, e1) in enumerate(ev):
                b = bufs[i % n_sets]
                e0.record(stream)
                if kind == "read":
                    sv.sv_stream_read(b, nbytes, sink, wgs, stream=stream)
                else:
                    sv.sv_stream_copy(b, b[half:], half, wgs, stream=stream)
                e1.record(stream)
            torch.cuda.synchronize()
            ms = statistics.mean(e0.elapsed_time(e1) for e0, e1 in ev[2:])
            if best is None or ms < best[0]:
                best = (ms, wgs)
        moved = nbytes if kind == "read" else 2 * half
        out[kind] = {"bytes": moved, "us": best[0] * 1e3, "GBps": moved / (best[0] * 1e-3) / 1e9, "workgroups": best[1]}
    return out


def bench_tconv(w, iters, sv, torch):
    """Mix-FFN temporal convolution (sv_tconv_block_step): the stream of w.n_blocks blocks enqueued back
    to back with the one-frame cache carried and committed after every block, `iters` passes between one
    event pair.  Its own roofline is the matrix cores' (2 * 3 * D * D flops per token)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    xs = [_randn_bf16((w.B, w.T, w.HW, w.D), gen) * 2.0 for _ in range(w.n_blocks)]       # ~N(0, 1)
    ys = [torch.empty_like(x) for x in xs]
    W = (_randn_bf16((3, w.D, w.D), gen).float() * (2.0 / (3 * w.D) ** 0.5)).to(torch.bfloat16)
    cache = torch.zeros((w.B, w.HW, w.D), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream()

    def run():
        for m in range(w.n_blocks):
            sv.sv_tconv_block_step(xs[m], W, cache if m else None, ys[m], cache, w.B, w.T, w.HW, w.D, stream=stream)

    for _ in range(max(2, iters // 2)):               # untimed passes: the first launches after idle run slower
        run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(iters):
        run()
    b.record(stream)
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / (iters * w.n_blocks)
    tflops = w.algorithmic_flops / us / 1e6

    # The same matrix-core instruction stream with nothing around it (sv_mfma_stream): as many workgroups as the
    # convolution has 256 x 256 tiles, each with the tile's K-steps; and 8 workgroups alone, for the clock an
    # almost idle device gives the same stream.
    tiles = -(-(w.B * w.T * w.HW) // 256) * -(-w.D // 256)
    k_steps = -(-3 * w.D // 32)
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")

    def stream_us(wgs):
        sv.sv_mfma_stream(wgs, k_steps, sink, stream=stream)
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(iters):
            sv.sv_mfma_stream(wgs, k_steps, sink, stream=stream)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / iters

    full_us, few_us = stream_us(tiles), stream_us(8)

    # The tile kernel with parts of its loop left out (sv_measure_tconv_variant), on the stream's first block:
    # what the loads into LDS and the operand reads from LDS cost on top of the matrix-core instructions.
    def variant_us(variant):
        for _ in range(2):
            sv.sv_measure_tconv_variant(variant, xs[0], W, None, ys[0], w.B, w.T, w.HW, w.D, stream=stream)
        a.record(stream)
        for _ in range(iters):
            sv.sv_measure_tconv_variant(variant, xs[0], W, None, ys[0], w.B, w.T, w.HW, w.D, stream=stream)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / iters

    loop_variants = None
    if w.D % 32 == 0:
        names = ["library kernel", "without the loads into LDS", "without the operand reads from LDS", "without both"]
        loop_variants = {names[v]: variant_us(v) for v in range(4)}
        loop_variants["library kernel, timed again"] = variant_us(0)
    wg_flops = k_steps * 4 * 32 * 2 * 32 * 32 * 16
    return {"workload": f"{w.name}: B={w.B} T={w.T} HW={w.HW} D={w.D}, {w.n_blocks} block(s)", "us_per_block": us,
            "tokens_per_s": w.tokens / (us * 1e-6), "dtype": "bf16",
            "roofline": {"bound": "mfma", "kernel": "tconv_mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                         "algorithmic_flops_per_launch": w.algorithmic_flops},
            "mfma_stream": {"what": "the tile loop's MFMAs alone, operands in registers, no LDS or memory traffic "
                                    "(sv_mfma_stream): one workgroup per tile, and 8 workgroups on an otherwise idle device",
                            "tiles": tiles, "k_steps": k_steps, "us": full_us,
                            "TFLOPs": tiles * wg_flops / full_us / 1e6,
                            "us_8_workgroups": few_us,
                            "us_per_tile_on_a_full_device": full_us / -(-tiles // 256), "us_per_tile_on_an_idle_device": few_us},
            "frac_of_mfma_stream": full_us / us,
            "loop_variants_us": loop_variants}


def bench_apply_variants(w, sets, steps, sv, torch):
    """The d = 64 apply kernel in its four forms (include/sv_measure.h: S in registers or in LDS, denominators
    through the matrix core or on the vector ALU), each timed between one event pair over `steps` launches on
    rotating buffer sets: the A/B figures behind two choices of the kernel design."""
    B, H, N, d = w.B, w.H, w.N, w.d
    S = torch.randn((B, H, d, d), dtype=torch.float32, device="cuda")
    z = torch.rand((B, H, d), dtype=torch.float32, device="cuda") * N * 0.2 + 1.0
    dsc = sv.desc_of(sets[0][0])
    stream = torch.cuda.current_stream()
    names = ["S in registers, denominators on the matrix core (the library's kernel)", "S in LDS, denominators on the matrix core",
             "S in registers, denominators on the vector ALU", "S in LDS, denominators on the vector ALU"]
    times = {v: [] for v in range(4)}
    for rnd in range(3):                                  # three rounds, the variants in a different order each
        for variant in [(rnd + k) % 4 for k in range(4)]:
            for i in range(3):
                q, _, _, o = sets[i % len(sets)]
                sv.sv_measure_apply_variant(variant, q, dsc, 0, N, S, z, w.eps, o, stream=stream)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record(stream)
            for i in range(steps):
                q, _, _, o = sets[i % len(sets)]
                sv.sv_measure_apply_variant(variant, q, dsc, 0, N, S, z, w.eps, o, stream=stream)
            b.record(stream)
            torch.cuda.synchronize()
            times[variant].append(a.elapsed_time(b) * 1e3 / steps)
    out = []
    for variant in range(4):
        us = statistics.median(times[variant])
        out.append({"variant": variant, "what": names[variant], "us_per_launch": us,
                    "hbm_frac": w.algorithmic_bytes / 2 / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS})
    return out


def cpu_baseline(w, sets, torch):
    """The float64 oracle on the host cores, on the full workload (one buffer set)."""
    import numpy as np
    from oracle import linattn_oracle as orc
    q, k, v, _ = sets[0]
    host = [t.view(torch.int16).cpu().numpy().view(np.uint16) for t in (q, k, v)]
    f32 = [(h.astype(np.uint32) << np.uint32(16)).view(np.float32) for h in host]   # exact widening
    best = None
    t_all = time.perf_counter()
    passes = 0
    while passes < 3 and (time.perf_counter() - t_all) < 30.0:
        t0 = time.perf_counter()
        orc.bidirectional(f32[0], f32[1], f32[2], w.eps)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
        passes += 1
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
    except OSError:
        pass
    return {"value": w.B * w.N / best, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"full {w.name} workload (B={w.B}, H={w.H}, N={w.N}, d={w.d}), best of {passes} passes, "
                      f"{best:.3f} s per pass, float64",
            "seconds_per_pass": best, "cpu_model": cpu_model}


def main():
    args = _parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path is one GPU's share of the layer); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2509_24695_amd as sv
    import sv_workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sv.load_library()              # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)

    from paper_2509_24695_amd.build import source_fingerprint
    fingerprint = source_fingerprint()
    table = measured_traffic()

    def headline_roofline(w, r, with_ceiling):
        """`roofline` of the slower kernel of the bidirectional step."""
        half = w.algorithmic_bytes / 2          # state reads K,V; apply reads Q and writes O
        dom = "state" if r["ms_state"] >= r["ms_apply"] else "apply"
        dom_ms_events = max(r["ms_state"], r["ms_apply"])
        # An event between two kernels adds a marker packet (2-3 us per kernel here).  The step time of the
        # timed region has no events inside it, so the event durations are scaled to add up to it: that is
        # the kernel's average launch duration in the timed region (rocprofv3's kernel trace agrees within 1 us).
        dom_ms = dom_ms_events * r["ms_per_step"] / (r["ms_state"] + r["ms_apply"])
        achieved = half / (dom_ms * 1e-3) / 1e9
        traffic, note = traffic_of(table, dom, w.name, fingerprint)
        roof = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": note,
                "algorithmic_bytes_per_launch": half, "avg_launch_ms": dom_ms,
                "avg_launch_ms_between_events": dom_ms_events}
        ceil = None
        if with_ceiling:
            ceil = bench_stream_ceiling(int(half), sv, torch)
            ref = ceil["read"] if dom == "state" else ceil["copy"]   # the state kernel only reads; the apply kernel reads and writes
            # both timed between events on the launch stream, the same way
            roof["frac_of_stream_ceiling"] = ref["us"] / (dom_ms_events * 1e3)
        return roof, ceil

    w = wl.workload(args.workload)
    r = bench_bidirectional(w, args.steps, args.warmup, args.sets, sv, torch)
    sec = r["ms_per_step"] * 1e-3
    roof, ceil = headline_roofline(w, r, not args.no_stream_ceiling)
    out = {
        "metric": "linear-attention tokens/s per layer (fwd)",
        "value": w.B * w.N / sec, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: bidirectional ReLU linear attention, B={w.B} H={w.H} N={w.N} d={w.d}, "
                               "bf16 tokens, fp32 state", "B": w.B, "H": w.H, "N": w.N, "d": w.d,
                   "buffer_sets": r["n_sets"]},
        "tflops": w.algorithmic_flops / sec / 1e12,
        "hbm_GBps_step": w.algorithmic_bytes / sec / 1e9,
        "hbm_frac_step": w.algorithmic_bytes / sec / 1e9 / HBM_PEAK_GBPS,
        "kernels_ms": {"state": r["ms_state"], "apply": r["ms_apply"],
                       "step_with_events": r["ms_per_step_with_events"]},
        "roofline": roof, "source_fingerprint": fingerprint,
    }
    if ceil:
        out["stream_ceiling"] = ceil
    if args.calibration_copy > 0:
        src = r["sets"][0][0]
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copy):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy"] = {"copies": args.calibration_copy, "bytes_read_each": src.numel() * 2,
                                   "bytes_written_each": src.numel() * 2}
    if not args.no_rope:
        # the same layer through the RoPE entry points (full equation of Sec. 3.2); the table
        # [N][d/2][2] fp32 is extra traffic (N*d*4 bytes per kernel, shared by the heads through L2)
        rr = bench_bidirectional(w, args.steps, args.warmup, 0, sv, torch, rope=_rope_table(w, torch),
                                 sets=r["sets"])
        out["rope_variant"] = {
            "ms_per_step": rr["ms_per_step"], "tokens_per_s": w.B * w.N / (rr["ms_per_step"] * 1e-3),
            "hbm_frac_step": w.algorithmic_bytes / (rr["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "kernels_ms": {"state": rr["ms_state"], "apply": rr["ms_apply"]},
        }
        # ... and with the rotation given as three per-axis tables that stay on chip
        rr = bench_bidirectional(w, args.steps, args.warmup, 0, sv, torch, rope=_rope_3d(w, torch, sv),
                                 sets=r["sets"])
        out["rope3d_variant"] = {
            "ms_per_step": rr["ms_per_step"], "tokens_per_s": w.B * w.N / (rr["ms_per_step"] * 1e-3),
            "hbm_frac_step": w.algorithmic_bytes / (rr["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "kernels_ms": {"state": rr["ms_state"], "apply": rr["ms_apply"]},
        }
    if not args.no_apply_variants and w.d == 64:
        out["apply_variants"] = bench_apply_variants(w, r["sets"], args.steps, sv, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, r["sets"], torch)
    del r
    torch.cuda.empty_cache()
    w480 = wl.workload("bidir_480p")
    if not args.no_secondary and w.name != w480.name:
        # the 480p-like layer (32 heads of 32 760 tokens), same protocol
        r1 = bench_bidirectional(w480, args.steps, args.warmup, 0, sv, torch)
        roof1, ceil1 = headline_roofline(w480, r1, not args.no_stream_ceiling)
        sec1 = r1["ms_per_step"] * 1e-3
        out["secondary"] = {
            "workload": f"{w480.name}: B={w480.B} H={w480.H} N={w480.N} d={w480.d}", "ms_per_step": r1["ms_per_step"],
            "tokens_per_s": w480.B * w480.N / sec1, "hbm_frac_step": w480.algorithmic_bytes / sec1 / 1e9 / HBM_PEAK_GBPS,
            "kernels_ms": {"state": r1["ms_state"], "apply": r1["ms_apply"]}, "roofline": roof1,
        }
        if ceil1:
            out["secondary"]["stream_ceiling"] = ceil1
        del r1
        torch.cuda.empty_cache()
    if not args.no_d112 and w.d == 64:
        # the 480p token grid in the paper's own head geometry (model-configuration table): H = 20, d = 112
        w2 = wl.workload("bidir_480p_h20d112")
        r2 = bench_bidirectional(w2, args.steps, args.warmup, 0, sv, torch)
        roof2, _ = headline_roofline(w2, r2, False)
        g = {"workload": f"{w2.name}: B={w2.B} H={w2.H} N={w2.N} d={w2.d}", "ms_per_step": r2["ms_per_step"],
             "tokens_per_s": w2.B * w2.N / (r2["ms_per_step"] * 1e-3),
             "hbm_frac_step": w2.algorithmic_bytes / (r2["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
             "kernels_ms": {"state": r2["ms_state"], "apply": r2["ms_apply"]}, "roofline": roof2}
        if not args.no_rope:
            for key, rope in (("rope", _rope_table(w2, torch)), ("rope3d", _rope_3d(w2, torch, sv))):
                r3 = bench_bidirectional(w2, args.steps, args.warmup, 0, sv, torch, rope=rope, sets=r2["sets"])
                g[key] = {"ms_per_step": r3["ms_per_step"],
                          "tokens_per_s": w2.B * w2.N / (r3["ms_per_step"] * 1e-3),
                          "hbm_frac_step": w2.algorithmic_bytes / (r3["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          "kernels_ms": {"state": r3["ms_state"], "apply": r3["ms_apply"]}}
        del r2
        torch.cuda.empty_cache()
        out["geometry_h20d112"] = g
    if not args.no_block_stream:
        cl = not args.no_stream_ceiling
        out["block_stream"] = [
            bench_block_stream(wl.workload("block_480p"), 10, sv, torch, ceiling=cl,
                               traffic=traffic_of(table, "block_step", "block_480p", fingerprint)),
            bench_block_stream(wl.workload("stream_720p"), args.stream_blocks, sv, torch, ceiling=cl,
                               traffic=traffic_of(table, "block_step", "stream_720p", fingerprint)),
        ]
        if not args.no_d112:
            out["block_stream"].append(bench_block_stream(wl.workload("block_480p_h20d112"), 10, sv, torch))
            if not args.no_rope:
                out["block_stream"].append(bench_block_stream(wl.workload("block_480p_h20d112"), 10, sv, torch,
                                                              rope=True))
                out["block_stream"].append(bench_block_stream(wl.workload("block_480p_h20d112"), 10, sv, torch,
                                                              rope="3d"))
        if not args.no_rope:
            out["block_stream"] += [
                bench_block_stream(wl.workload("block_480p"), 10, sv, torch, rope=True),
                bench_block_stream(wl.workload("stream_720p"), args.stream_blocks, sv, torch, rope=True),
                bench_block_stream(wl.workload("block_480p"), 10, sv, torch, rope="3d"),
                bench_block_stream(wl.workload("stream_720p"), args.stream_blocks, sv, torch, rope="3d"),
            ]
    if not args.no_tconv:
        # the other cached operator of the block-causal model (Sec. 3.3.1): dense, so bound by the matrix cores
        out["tconv"] = [bench_tconv(wl.TCONV_WORKLOADS["tconv_480p"], 10, sv, torch),
                        bench_tconv(wl.TCONV_WORKLOADS["tconv_block_480p"], 10, sv, torch)]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
