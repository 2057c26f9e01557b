#!/usr/bin/env python3
"""Benchmark of the RaZeR W4A16 / W4A4 linear path on one MI355X.

Headline: HBM GB/s of the fused-decode GEMV at M=1 over a
Llama-7B-shaped decoder layer (q,k,v,o 4096x4096; gate,up 11008x4096; down
4096x11008), weights resident in HBM in RaZeR form.  One timed "step" is one
pass over the seven projections at M=1; enough distinct copies of the packed
layer are rotated through that every pass streams its weights from HBM rather
than from the last-level cache.  The other legs of the path (small-M GEMV,
MFMA GEMM at M=512/2048, encoder, decoder, W4A4) are timed in the same run and
reported in "legs".  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
LLC_BYTES = 256 << 20          # Infinity Cache
# HBM bytes per {gate,up} launch come from the FETCH_SIZE / WRITE_SIZE counter runs summarised in this file
# (counters cannot be read live); bench.py only parses the figure out of it
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemv_m1_llama7b_hbm_traffic.txt")


def profiled_traffic_bytes():
    """`gate_up_hbm_bytes_per_launch = N` from the committed counter summary, or None."""
    import re
    try:
        m = re.search(r"gate_up_hbm_bytes_per_launch\s*=\s*([0-9,]+)", open(TRAFFIC_PROFILE).read())
        return int(m.group(1).replace(",", "")) if m else None
    except OSError:
        return None


def profiled_trace_avg_us():
    """`gate_up_trace_avg_us = T` from the committed kernel-trace summary (a profiled run of this command), or None."""
    import re
    try:
        m = re.search(r"gate_up_trace_avg_us\s*=\s*([0-9.]+)", open(os.path.join(ROOT, "profiles", "gemv_m1_llama7b_kernel_stats.txt")).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--legs", default="all", help="all | gemv (headline only) | gemm (headline + the M=2048 GEMM leg)")
    p.add_argument("--ramp-ms", type=float, default=250.0,
                   help="untimed load before every measurement, so it runs at sustained clocks (short for profiler runs)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying HIP graphs")
    return p.parse_args()


def student_t_weight(n, k, gen, outlier_frac=0.001, gain=20.0):
    """fp32 [n][k] on the GPU: Student-t(nu=4) scaled to std 0.02, 0.1% of input channels x20."""
    import torch
    z = torch.randn((n, k), generator=gen, device="cuda", dtype=torch.float32)
    chi = torch.zeros((n, k), device="cuda", dtype=torch.float32)
    for _ in range(4):
        chi += torch.randn((n, k), generator=gen, device="cuda", dtype=torch.float32) ** 2
    w = z / torch.sqrt(chi / 4.0) * (0.02 / 2.0 ** 0.5)
    n_out = int(round(outlier_frac * k))
    if n_out:
        cols = torch.randperm(k, generator=gen, device="cuda")[:n_out]
        w[:, cols] *= gain
    return w


RAMP_S = 0.25                  # untimed load before every measurement (see time_region)


def time_region(fn, steps, warmup, graph_period=0):
    """Run fn(step) warmup+steps times on the current stream; returns ms per step (HIP events).

    Before the warm-up steps the same fn runs untimed for RAMP_S seconds: after any idle or
    host-bound phase (set-up, allocation, the previous leg's teardown) this GPU takes tens of
    milliseconds of load to return to its sustained clocks, and a short region measured from idle
    reads 10-13 % slow (measured: 37.3 us vs 33.0 us per M=1 step).  The timed region is still
    exactly `steps` steps after `warmup` warm-up steps.

    graph_period > 0: fn(i) only depends on i % graph_period; each of those variants is captured
    once into a HIP graph (the launches go to the capturing stream through the C ABI) and the
    timed region replays the graphs, so the host cost of the Python binding is off the clock."""
    import torch
    if graph_period:
        graphs = []
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for i in range(graph_period):
                fn(i)                                   # warm up outside capture
            torch.cuda.synchronize()
            for i in range(graph_period):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    fn(i)
                graphs.append(g)
        torch.cuda.synchronize()
        eager = fn
        fn = lambda i: graphs[i % graph_period].replay()
    t0, j = time.perf_counter(), 0
    while time.perf_counter() - t0 < RAMP_S:
        for _ in range(8):
            fn(j)
            j += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_dispatches(fn, n, warmup):
    """Average duration (ms) of single dispatches of the ONE kernel fn(i) launches: the library records
    the begin and end time stamps of the dispatch itself into a HIP event pair handed to it through
    razer_probe_dispatch_events -- the per-dispatch duration a kernel trace (rocprofv3 --kernel-trace)
    reports, measured live on the stream the kernel runs on.  Every launch has its own pair; all pairs
    are read after one final synchronize.  Returns (mean, median)."""
    import torch
    import paper_2501_04052_amd as razer
    t0, j = time.perf_counter(), 0
    while time.perf_counter() - t0 < RAMP_S:
        for _ in range(8):
            fn(j)
            j += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        fn(i)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for e0, e1 in pairs:                              # a first record creates the HIP event handles
        e0.record()
        e1.record()
    torch.cuda.synchronize()
    try:
        for i, (e0, e1) in enumerate(pairs):
            razer.razer_probe_dispatch_events(e0, e1)
            fn(warmup + i)
    finally:
        razer.razer_probe_dispatch_events(None, None)
    torch.cuda.synchronize()
    d = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)
    return sum(d) / n, d[n // 2]


def main():
    global RAMP_S
    args = parse()
    RAMP_S = args.ramp_ms / 1e3
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2501_04052_amd as razer
    from paper_2501_04052_amd import binding, synth

    razer.load_library()            # raises if the HIP library is not built: no fallback
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2000)
    layers = synth.LLAMA_7B_LAYER
    sv = (5.0, 8.0)

    # ---- encode the layer once (also the encoder leg) --------------------------------
    legs = {}
    packed = []
    enc_bytes = enc_ms = 0.0
    for name, n, k in layers:
        w = student_t_weight(n, k, gen)
        t = razer.razer_quantize(w, razer.WEIGHT, sv)                      # warm-up + result
        torch.cuda.synchronize()
        ms = time_region(lambda i: razer.razer_quantize(w, razer.WEIGHT, sv, out=t), 3, 1)
        enc_ms += ms
        enc_bytes += n * k * (4 + 0.5625)
        packed.append(t)
        del w
    legs["encode_weights_fp32"] = {"GB/s": enc_bytes / enc_ms / 1e6, "ms_per_layer_set": enc_ms,
                                   "bytes": "4 B in + 0.5625 B out per element; the absmax pre-pass re-reads the input"}

    layer_bytes = sum(n * k * 9 // 16 for _, n, k in layers)
    n_copies = max(2, -(-2 * LLC_BYTES // layer_bytes))                     # working set >= 2x the LLC
    copies = [packed]
    for _ in range(n_copies - 1):
        copies.append([razer.RazerTensor(t.codes.clone(), t.scales.clone(), t.tensor_scale.clone(),
                                         t.rows, t.cols, t.fmt, t.sv) for t in packed])

    def make_act(m, k, seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        return torch.randn((m, k), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)

    packed_copies = []                                              # the private interleaved layout, built on first use

    def linear_leg(m, steps, warmup, rotate=True, graph=False, grouped=False, prepared=False, prepared_single=False,
                   prepacked=False):
        if prepacked and not packed_copies:
            packed_copies.extend([[razer.razer_prepack(t) for t in cp] for cp in copies])
        src_copies = packed_copies if prepacked else copies
        acts = {k: make_act(m, k, 2100 + m) for k in {k for _, _, k in layers}}
        outs = [torch.empty((m, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in layers]
        plans = None
        if prepared_single:
            # seven prepared razer_linear calls per step (workspaces allocated once, not per call)
            prepared = True
            plans = [[razer.prepare_linear(t, acts[t.cols], outs[j]) for j, t in enumerate(cp)] for cp in copies]
            stream = torch.cuda.current_stream().cuda_stream
        if prepared and plans is None:
            # the marshalled C-ABI calls are built once per packed copy and re-issued every step:
            # plain launches on torch's current stream, no graph, no per-call Python marshalling
            plans = [[razer.prepare_linear_grouped(cp[0:3], acts[cp[0].cols], outs[0:3]),
                      razer.prepare_linear(cp[3], acts[cp[3].cols], outs[3]),
                      razer.prepare_linear_grouped(cp[4:6], acts[cp[4].cols], outs[4:6]),
                      razer.prepare_linear(cp[6], acts[cp[6].cols], outs[6])] for cp in src_copies]
            stream = torch.cuda.current_stream().cuda_stream

        def step(i):
            if prepared:
                for call in plans[i % n_copies if rotate else 0]:
                    call(stream)
                return
            cp = copies[i % n_copies] if rotate else copies[0]
            if grouped:
                # the projections that consume the same activation go out as one launch each:
                # {q,k,v}, o, {gate,up}, down -- the dependency structure of a decoder layer
                razer.razer_linear_grouped(cp[0:3], acts[cp[0].cols], outs=outs[0:3])
                razer.razer_linear(cp[3], acts[cp[3].cols], out=outs[3])
                razer.razer_linear_grouped(cp[4:6], acts[cp[4].cols], outs=outs[4:6])
                razer.razer_linear(cp[6], acts[cp[6].cols], out=outs[6])
                return
            for j, t in enumerate(cp):
                razer.razer_linear(t, acts[t.cols], out=outs[j])
        ms = time_region(step, steps, warmup, graph_period=(n_copies if rotate else 1) if graph else 0)
        byts = sum(n * k * 9 // 16 + 2 * m * k + 2 * m * n + 4 for _, n, k in layers)
        flops = sum(2.0 * m * n * k for _, n, k in layers)
        return ms, byts, flops

    # ---- headline: GEMV at M=1 ----------------------------------------------------------
    use_graph = not args.no_graph
    ms1, bytes1, _ = linear_leg(1, args.steps, args.warmup, grouped=True, prepared=True)
    gbs = bytes1 / ms1 / 1e6
    quarter = max(10, args.steps // 4)
    if use_graph:
        msg, _, _ = linear_leg(1, quarter, 5, graph=True, grouped=True)
        legs["gemv_m1_graph_replay"] = {"GB/s": bytes1 / msg / 1e6, "ms_per_step": msg,
                                        "note": "same step captured once per packed copy into a HIP graph and replayed"}
    ms1s, _, _ = linear_leg(1, quarter, 5, graph=use_graph)
    legs["gemv_m1_seven_launches"] = {"GB/s": bytes1 / ms1s / 1e6, "ms_per_step": ms1s,
                                      "note": "same step as seven razer_linear calls instead of four (no grouping)"}
    ms1c, _, _ = linear_leg(1, quarter, 5, rotate=False, grouped=True, prepared=True)
    legs["gemv_m1_cache_resident"] = {"GB/s": bytes1 / ms1c / 1e6, "note": "same 113.8 MB copy every step: served by the last-level cache, not HBM"}
    ms1p, _, _ = linear_leg(1, args.steps, args.warmup, grouped=True, prepared=True, prepacked=True)
    legs["gemv_m1_prepacked_layout"] = {
        "GB/s": bytes1 / ms1p / 1e6, "frac_hbm": bytes1 / ms1p / 1e6 / HBM_PEAK_GBS, "ms_per_step": ms1p,
        "note": "same step on weights repacked offline with razer_prepack (scale bytes interleaved with their 2048-element "
                "code runs; results bit-identical); algorithmic bytes as in the headline, the padding of short runs is never read"}
    if args.legs != "all":
        packed_copies.clear()
    ms1e, _, _ = linear_leg(1, quarter, 5, grouped=True)
    legs["gemv_m1_unprepared_calls"] = {"GB/s": bytes1 / ms1e / 1e6, "ms_per_step": ms1e,
                                        "note": "same step with the Python binding marshalling every call (host-bound)"}

    # dominant kernel of the step: the {gate, up} launch (gemv_stream_grouped_kernel<1,2,2,2,2,false,0>, 44 % of
    # the step's bytes).  Two live figures, both with HIP events on the stream it runs on:
    #   per dispatch  -- begin/end time stamps of each single dispatch (what a kernel trace reports; the
    #                    `roofline` entry uses this one, so it can be recomputed from profiles/)
    #   back to back  -- a region of launches of that kernel alone, region time / launches (in a stream the
    #                    drain of one launch overlaps the ramp-up of the next, so this reads lower)
    a1 = make_act(1, 4096, 2101)
    o2 = [torch.empty((1, 11008), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    dom = [razer.prepare_linear_grouped(cp[4:6], a1, o2) for cp in copies]
    dstream = torch.cuda.current_stream().cuda_stream
    dom_stream_ms = time_region(lambda i: dom[i % n_copies](dstream), max(100, args.steps), 20)
    dom_ms, dom_median_ms = time_dispatches(lambda i: dom[i % n_copies](dstream), max(200, args.steps), 20)
    dom_bytes = 2 * (11008 * 4096 * 9 // 16 + 2 * 11008 + 4) + 2 * 4096
    # per-dispatch durations of the step's four launches, measured the same way
    acts1 = {k: make_act(1, k, 2101) for k in (4096, 11008)}
    outs1 = [torch.empty((1, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in layers]
    per_launch = {}
    for label, mk, byts in (
            ("qkv", lambda cp: razer.prepare_linear_grouped(cp[0:3], acts1[4096], outs1[0:3]),
             3 * (4096 * 4096 * 9 // 16 + 2 * 4096 + 4) + 2 * 4096),
            ("o", lambda cp: razer.prepare_linear(cp[3], acts1[4096], outs1[3]), 4096 * 4096 * 9 // 16 + 4 * 4096 + 4),
            ("down", lambda cp: razer.prepare_linear(cp[6], acts1[11008], outs1[6]),
             4096 * 11008 * 9 // 16 + 2 * 11008 + 2 * 4096 + 4)):
        calls = [mk(cp) for cp in copies]
        mean_ms, _ = time_dispatches(lambda i: calls[i % n_copies](dstream), 100, 10)
        per_launch[label] = {"us": mean_ms * 1e3, "GB/s": byts / mean_ms / 1e6}
    per_launch["gate_up"] = {"us": dom_ms * 1e3, "GB/s": dom_bytes / dom_ms / 1e6}
    legs["gemv_m1_per_dispatch"] = per_launch

    # measured ceilings, timed in this run: a kernel that only streams a buffer of the size of a launch's
    # weights (rotated through a pool larger than the last-level cache), per dispatch and back to back
    pool = torch.empty(3 * LLC_BYTES, dtype=torch.uint8, device="cuda")
    pool.random_(0, 256, generator=gen)
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    ceil = {}
    for label, size in (("9.4MB", 4096 * 4096 * 9 // 16), ("25.4MB", 4096 * 11008 * 9 // 16), ("28.3MB", 3 * 4096 * 4096 * 9 // 16),
                        ("50.8MB", dom_bytes), ("264MB", 2 * 28672 * 8192 * 9 // 16)):
        size = size // 4096 * 4096
        slots = [pool[o:o + size] for o in range(0, pool.numel() - size + 1, size)]
        best = None
        for wgs in (1024, 2048, 4096, 8192, 16384):
            fn = lambda i: razer.razer_probe_stream_read(slots[i % len(slots)], wgs, sink)
            b2b = time_region(fn, 60, 10)
            if best is None or b2b < best[1]:
                best = (wgs, b2b)
        wgs = best[0]
        fn = lambda i: razer.razer_probe_stream_read(slots[i % len(slots)], wgs, sink)
        disp, _ = time_dispatches(fn, 100, 10)
        ceil[label] = {"bytes": size, "workgroups": wgs, "per_dispatch_us": disp * 1e3, "per_dispatch_GB/s": size / disp / 1e6,
                       "back_to_back_us": best[1] * 1e3, "back_to_back_GB/s": size / best[1] / 1e6}
    del pool, slots
    # the M=1 step made of four load-only kernels of the sizes of its four launches ({q,k,v}, o, {gate,up}, down):
    # what a sequence of four dependent launches that only read their weights would reach
    step_ceiling_us = sum(ceil[lab]["per_dispatch_us"] for lab in ("28.3MB", "9.4MB", "50.8MB", "25.4MB"))
    ceil["step_of_four_load_only_kernels"] = {"us": step_ceiling_us, "GB/s": bytes1 / step_ceiling_us / 1e3,
                                              "frac_hbm": bytes1 / step_ceiling_us / 1e3 / HBM_PEAK_GBS}
    legs["ceiling_stream_read"] = ceil
    fl_box = [0.0]

    def mfma_fn(i):
        fl_box[0] = razer.razer_probe_mfma_bf16(4000, 512, sink)
    mfma_ms = time_region(mfma_fn, 10, 2)
    legs["ceiling_mfma_bf16_loop"] = {"TFLOP/s": fl_box[0] / mfma_ms / 1e9, "ms": mfma_ms,
                                      "note": "register-resident v_mfma_f32_32x32x16_bf16 loop, 2 wavefronts per SIMD, no memory "
                                              "traffic, operands with well-mixed bits (the sustained clock depends on them)"}

    def fp4_fn(i):
        fl_box[0] = razer.razer_probe_mfma_fp4(2000, 512, sink)
    fp4_ms = time_region(fp4_fn, 10, 2)
    legs["ceiling_mfma_fp4_scaled_loop"] = {
        "TFLOP/s": fl_box[0] / fp4_ms / 1e9, "ms": fp4_ms,
        "note": "register-resident v_mfma_scale_f32_32x32x64_f8f6f4 loop, FP4 x FP4 with E8M0 scales: context for the two-pass "
                "FP4 realisation of W4A4 (App. D.3), which this GPU's power-of-two scales per 32 elements cannot carry exactly"}

    gemm_roof = None

    def gemm_leg(m):
        # {q,k,v}, o, {gate,up}, down as four prepared calls, like the decode step
        ms, _, fl = linear_leg(m, 5, 2, prepared=True)
        legs["gemm_m%d" % m] = {"TFLOP/s": fl / ms / 1e9, "frac_mfma_bf16": fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                "ms_per_step": ms}
        return ms, fl

    def gemm_roofline(ms, fl):
        # dominant kernel of the M=2048 layer: the {gate,up} launch (gemm_rb_grouped_kernel), per dispatch
        m = 2048
        a2k = make_act(m, 4096, 2100 + m)
        o2k = [torch.empty((m, 11008), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
        calls = [razer.prepare_linear_grouped(cp[4:6], a2k, o2k) for cp in copies]
        st = torch.cuda.current_stream().cuda_stream
        dms, _ = time_dispatches(lambda i: calls[i % n_copies](st), 20, 3)
        dfl = 2.0 * m * 2 * 11008 * 4096
        return {"bound": "mfma", "achieved": dfl / dms / 1e9, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": dfl / dms / 1e9 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                "kernel": "gemm_rb_grouped_kernel<4,2,1,8,false> on {gate,up} 2 x 11008x4096 at M=2048 (44 % of the layer's flops), "
                          "flops = 2MNK, per-dispatch duration from the dispatch's own time stamps",
                "avg_dispatch_us": dms * 1e3, "flops_per_launch": dfl,
                "layer_TFLOP/s": fl / ms / 1e9, "layer_frac": fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                "layer_note": "Llama-7B layer set at M=2048 as 4 calls, whole-leg time",
                "measured_ceiling_TFLOP/s": legs.get("ceiling_mfma_bf16_loop", {}).get("TFLOP/s")}

    if args.legs == "gemm":                                  # profiler runs: only the M=2048 GEMM leg
        gemm_roof = gemm_roofline(*gemm_leg(2048))
    if args.legs == "all":
        for m in (4, 16):
            ms, b, _ = linear_leg(m, max(10, args.steps // 4), 5, prepared=True)
            legs["linear_m%d" % m] = {"GB/s": b / ms / 1e6, "frac_hbm": b / ms / 1e6 / HBM_PEAK_GBS, "ms_per_step": ms}
        ms, b, _ = linear_leg(4, max(10, args.steps // 4), 5, prepared=True, prepacked=True)
        legs["linear_m4_prepacked_layout"] = {"GB/s": b / ms / 1e6, "frac_hbm": b / ms / 1e6 / HBM_PEAK_GBS, "ms_per_step": ms}
        packed_copies.clear()
        # the batch curve between the decode regime and the large GEMMs: four prepared calls per step
        for m in (64, 128, 256):
            ms, _, fl = linear_leg(m, 10, 3, prepared=True)
            legs["linear_m%d" % m] = {"TFLOP/s": fl / ms / 1e9, "ms_per_step": ms, "us_per_row": ms * 1e3 / m}
        for m in (512, 2048):
            ms, fl = gemm_leg(m)
            ms7, _, _ = linear_leg(m, 5, 2, prepared_single=True)
            legs["gemm_m%d_seven_calls" % m] = {"TFLOP/s": fl / ms7 / 1e9, "ms_per_step": ms7}
            if m == 2048:
                gemm_roof = gemm_roofline(ms, fl)
        # context, not product: the vendor library's dense bf16 GEMM (torch.matmul -> hipBLASLt) on the same
        # seven shapes at M=2048 with already-decoded bf16 weights, i.e. the same contraction with no decode
        dense_w = {(n, k): torch.randn((n, k), generator=gen, device="cuda").to(torch.bfloat16) * 0.02
                   for n, k in {(n, k) for _, n, k in layers}}
        dense_a = {k: make_act(2048, k, 2100 + 2048) for k in {k for _, _, k in layers}}

        def dense_step(i):
            for _, n, k in layers:
                torch.matmul(dense_a[k], dense_w[(n, k)].t())
        ms = time_region(dense_step, 5, 2)
        fl = sum(2.0 * 2048 * n * k for _, n, k in layers)
        legs["dense_bf16_library_gemm_m2048"] = {
            "TFLOP/s": fl / ms / 1e9, "ms_per_step": ms,
            "note": "reference only: torch.matmul (hipBLASLt) on bf16 weights of the same shapes, no decode, 7 calls"}
        del dense_w, dense_a
        # decoder leg: packed -> bf16
        t = packed[4]
        out = torch.empty((t.rows, t.cols), dtype=torch.bfloat16, device="cuda")
        ms = time_region(lambda i: razer.razer_dequant(t, out=out), 10, 2)
        legs["dequant_bf16_11008x4096"] = {"GB/s": t.rows * t.cols * (0.5625 + 2) / ms / 1e6}
        del out
        # W4A4 leg: on-the-fly activation encode + linear against the gate projection
        a = make_act(4096, 4096, 5000)
        cols = torch.randperm(4096, generator=gen, device="cuda")[:20]
        a[:, cols] *= 50.0
        aq = razer.razer_quantize(a, razer.ACT, (5.0, 0.0))
        ms_e = time_region(lambda i: razer.razer_quantize(a, razer.ACT, (5.0, 0.0), out=aq), 10, 2)
        y = torch.empty((4096, 11008), dtype=torch.bfloat16, device="cuda")
        # with the workspace the W4A4 query asks for (the library then decodes the activations once and runs the
        # weight-only path), and with a token workspace (the single fused kernel that decodes both operands per tile)
        ws_big = torch.empty(razer.razer_workspace_bytes(binding.OP_LINEAR_W4A4, 11008, 4096, 4096), dtype=torch.uint8, device="cuda")
        ws_small = torch.empty(256, dtype=torch.uint8, device="cuda")
        ms_l = time_region(lambda i: razer.razer_linear(packed[4], aq, out=y, workspace=ws_big), 5, 2)
        ms_f = time_region(lambda i: razer.razer_linear(packed[4], aq, out=y, workspace=ws_small), 5, 2)
        legs["w4a4_act_encode_4096x4096"] = {"GB/s": 4096 * 4096 * (2 + 0.5625) / ms_e / 1e6, "ms": ms_e}
        legs["w4a4_linear_4096x11008x4096"] = {"TFLOP/s": 2.0 * 4096 * 11008 * 4096 / ms_l / 1e9, "ms": ms_l,
                                               "end_to_end_TFLOP/s": 2.0 * 4096 * 11008 * 4096 / (ms_l + ms_e) / 1e9,
                                               "fused_kernel_TFLOP/s": 2.0 * 4096 * 11008 * 4096 / ms_f / 1e9}
        del ws_big, ws_small
        # the same layer in the decode regime: few activation rows, RaZeR activations (both forms as above)
        for mm in (1, 16):
            am = make_act(mm, 4096, 5100 + mm)
            aqm = razer.razer_quantize(am, razer.ACT, (5.0, 0.0))
            ym = torch.empty((mm, 11008), dtype=torch.bfloat16, device="cuda")
            wsm = torch.empty(razer.razer_workspace_bytes(binding.OP_LINEAR_W4A4, 11008, 4096, mm), dtype=torch.uint8, device="cuda")
            wsf = torch.empty(max(256, razer.razer_workspace_bytes(binding.OP_LINEAR, 11008, 4096, mm)), dtype=torch.uint8, device="cuda")
            gates = [cp[4] for cp in copies]
            ms_s = time_region(lambda i: razer.razer_linear(gates[i % n_copies], aqm, out=ym, workspace=wsm), 50, 10)
            ms_f = time_region(lambda i: razer.razer_linear(gates[i % n_copies], aqm, out=ym, workspace=wsf), 20, 5)
            legs["w4a4_linear_m%d_11008x4096" % mm] = {"us": ms_s * 1e3, "fused_kernel_us": ms_f * 1e3,
                                                        "note": "unprepared binding calls (host cost included)"}
            del wsm, wsf

    # ---- Llama-70B-shaped layer (configs[3]): 481 MB of packed weights, far beyond the LLC ----
    if args.legs == "all":
        del copies
        torch.cuda.empty_cache()
        big = []
        g70 = torch.Generator(device="cuda")
        g70.manual_seed(4000)
        for name, n, k in synth.LLAMA_70B_LAYER:
            # random packed codes / scale bytes: the kernels' speed does not depend on the values
            codes = torch.randint(0, 256, (n, k // 2), generator=g70, device="cuda", dtype=torch.uint8)
            scales = torch.randint(0, 256, (n, k // 16), generator=g70, device="cuda", dtype=torch.uint8)
            big.append(razer.RazerTensor(codes, scales, torch.tensor([1e-3], device="cuda"), n, k, razer.WEIGHT, sv))
        bytes70 = sum(n * k * 9 // 16 for _, n, k in synth.LLAMA_70B_LAYER)
        for m in (1, 8):
            acts = {k: make_act(m, k, 4100 + m) for k in {k for _, _, k in synth.LLAMA_70B_LAYER}}
            outs = [torch.empty((m, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in synth.LLAMA_70B_LAYER]
            plans70 = [razer.prepare_linear_grouped(big[0:3], acts[8192], outs[0:3]),
                       razer.prepare_linear(big[3], acts[8192], outs[3]),
                       razer.prepare_linear_grouped(big[4:6], acts[8192], outs[4:6]),
                       razer.prepare_linear(big[6], acts[28672], outs[6])]
            st70 = torch.cuda.current_stream().cuda_stream

            def step70(i):
                for call in plans70:
                    call(st70)
            ms = time_region(step70, 20, 3)
            b = bytes70 + sum(2 * m * k + 2 * m * n + 4 for _, n, k in synth.LLAMA_70B_LAYER)
            legs["llama70b_layer_m%d" % m] = {"GB/s": b / ms / 1e6, "frac_hbm": b / ms / 1e6 / HBM_PEAK_GBS,
                                             "ms_per_step": ms, "note": "configs[3]: 481 MB packed layer, one pass"}
        # the same layer at M=4096 (prefill): 7.0 TFLOP per pass
        m = 4096
        acts = {k: make_act(m, k, 4100 + m) for k in {k for _, _, k in synth.LLAMA_70B_LAYER}}
        outs = [torch.empty((m, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in synth.LLAMA_70B_LAYER]
        plans70 = [razer.prepare_linear_grouped(big[0:3], acts[8192], outs[0:3]),
                   razer.prepare_linear(big[3], acts[8192], outs[3]),
                   razer.prepare_linear_grouped(big[4:6], acts[8192], outs[4:6]),
                   razer.prepare_linear(big[6], acts[28672], outs[6])]

        def step70p(i):
            for call in plans70:
                call(st70)
        ms = time_region(step70p, 3, 1)
        fl = sum(2.0 * m * n * k for _, n, k in synth.LLAMA_70B_LAYER)
        legs["llama70b_layer_m4096"] = {"TFLOP/s": fl / ms / 1e9, "frac_mfma_bf16": fl / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                                        "ms_per_step": ms, "note": "configs[3] at M=4096, 4 calls"}
        del big, plans70, acts, outs

    # ---- block sizes 32, 64, 128 (the paper's block-size study): M=1 decode step, 4 launches -------
    if args.legs == "all":
        torch.cuda.empty_cache()
        for block in (32, 64, 128, "f16"):
            # "f16": the paper's own kernel format -- blocks of 128 with one FP16 scale word
            f16 = block == "f16"
            if f16:
                block = 128
            gb = torch.Generator(device="cuda")
            gb.manual_seed(6000 + block + f16)
            sets = []
            for _ in range(n_copies):
                ts1 = torch.tensor([1e-3], device="cuda")
                sets.append([razer.RazerTensor(
                    torch.randint(0, 256, (n, k // 2), generator=gb, device="cuda", dtype=torch.uint8),
                    torch.randint(0, 256, (n, k // block * (2 if f16 else 1)), generator=gb, device="cuda", dtype=torch.uint8),
                    ts1, n, k, razer.WEIGHT_F16 if f16 else razer.WEIGHT, sv, block) for _, n, k in layers])
            acts = {k: make_act(1, k, 2101) for k in {k for _, _, k in layers}}
            outs = [torch.empty((1, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in layers]
            # the same 4 launches as the headline leg: {q,k,v}, o, {gate,up}, down
            plans = [[razer.prepare_linear_grouped(cp[0:3], acts[cp[0].cols], outs[0:3]),
                      razer.prepare_linear(cp[3], acts[cp[3].cols], outs[3]),
                      razer.prepare_linear_grouped(cp[4:6], acts[cp[4].cols], outs[4:6]),
                      razer.prepare_linear(cp[6], acts[cp[6].cols], outs[6])] for cp in sets]
            stream = torch.cuda.current_stream().cuda_stream

            def stepb(i):
                for call in plans[i % n_copies]:
                    call(stream)
            ms = time_region(stepb, max(10, args.steps // 4), 5)
            sbytes = 2 if f16 else 1
            b = sum(n * k // 2 + n * k // block * sbytes + 2 * k + 2 * n + 4 for _, n, k in layers)
            legs["gemv_m1_block128_fp16_scale" if f16 else "gemv_m1_block%d" % block] = {
                "GB/s": b / ms / 1e6, "ms_per_step": ms, "bits_per_weight": 4 + 8.0 * sbytes / block,
                "note": "same layer shapes with %d-element blocks%s, random packed bytes, 4 launches"
                        % (block, " and one FP16 scale word per block (the format of the paper's own kernel)" if f16 else "")}
            if f16:
                # the same format beyond the decode regime: matrix-core kernel with per-block folds
                for mm in (16, 64, 2048):
                    actm = {k: make_act(mm, k, 2100 + mm) for k in {k for _, _, k in layers}}
                    outm = [torch.empty((mm, n), dtype=torch.bfloat16, device="cuda") for _, n, _ in layers]
                    # the same 4 calls as every other leg ({q,k,v} and {gate,up} through razer_linear_grouped, which is
                    # one launch each up to 32 rows and the sequence of single calls beyond)
                    plansm = [[razer.prepare_linear_grouped(cp[0:3], actm[cp[0].cols], outm[0:3]),
                               razer.prepare_linear(cp[3], actm[cp[3].cols], outm[3]),
                               razer.prepare_linear_grouped(cp[4:6], actm[cp[4].cols], outm[4:6]),
                               razer.prepare_linear(cp[6], actm[cp[6].cols], outm[6])] for cp in sets]

                    def stepm(i):
                        for call in plansm[i % n_copies]:
                            call(stream)
                    msm = time_region(stepm, 5, 2)
                    flm = sum(2.0 * mm * n * k for _, n, k in layers)
                    legs["linear_m%d_block128_fp16_scale" % mm] = {
                        "TFLOP/s": flm / msm / 1e9, "ms_per_step": msm,
                        "note": "bare FP4 operands on the matrix cores, each 128-element block's partial sums folded with its "
                                "FP16 scale in fp32: K-in-workgroup kernel up to 64 rows, LDS-staged tiled kernels beyond"}
                    del plansm, actm, outm
            del sets, plans
            torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle, as it stands, on the host cores ------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        name, n, k = layers[0]
        rows = 1024                                                     # bounded sample: 1024 output rows of q
        t = packed[0]
        wq = (t.codes[:rows].cpu().numpy(), t.scales[:rows].cpu().numpy(),
              np.float32(t.tensor_scale.cpu().numpy()[0]))
        a_bits = make_act(1, k, 2101).view(torch.int16).cpu().numpy().view(np.uint16)
        oracle.linear(wq, a_bf16=a_bits, rows=None, cols=np.arange(8, dtype=np.int64))   # page in
        nthreads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count()))
        sample_bytes = rows * k * 9 // 16 + 2 * k + 2 * rows

        def timed(threads, seconds):
            oracle.set_threads(threads)
            t0 = time.perf_counter()
            reps = 0
            while time.perf_counter() - t0 < seconds:
                oracle.linear(wq, a_bf16=a_bits)
                reps += 1
            return (time.perf_counter() - t0) / reps, reps
        dt_omp, reps_omp = timed(nthreads, 8.0)
        dt_one, reps_one = timed(1, 8.0)
        oracle.set_threads(nthreads)
        cpu = {"value": sample_bytes / dt_omp / 1e9, "unit": "GB/s", "cores": nthreads, "kind": "oracle",
               "sample": "oracle_linear, M=1, first %d of %d output rows of the %dx%d q projection, %d repeats in ~8 s "
                         "with OpenMP over the output rows" % (rows, n, n, k, reps_omp),
               "single_thread": {"value": sample_bytes / dt_one / 1e9, "unit": "GB/s", "cores": 1,
                                 "sample": "the same sample on one thread, %d repeats in ~8 s" % reps_one}}

    trace_us = profiled_trace_avg_us()
    out = {
        "metric": "RaZeR W4A16 GEMV HBM GB/s at M=1 (Llama-7B-shaped layer set)",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-7B-shaped decoder layer (q,k,v,o 4096x4096; gate,up 11008x4096; "
                               "down 4096x11008), RaZeR weights (block 16, E3M3 scale + 2 meta bits, sv {5,8}), M=1; "
                               "one step = the 7 projections once, as 4 launches: {q,k,v} and {gate,up} share their activation and go through "
                               "razer_linear_grouped; plain stream launches through the C ABI; %d packed copies rotated (%.0f MB > 2x LLC); "
                               "fp4 codes x bf16 activations, fp32 accumulate" % (n_copies, n_copies * layer_bytes / 1e6),
                   "m": 1, "bytes_per_step": bytes1},
        "roofline": {"bound": "hbm", "achieved": dom_bytes / dom_ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": dom_bytes / dom_ms / 1e6 / HBM_PEAK_GBS, "traffic": profiled_traffic_bytes(),
                     "kernel": "gemv_stream_grouped_kernel<1,2,2,2,2,false,0> on {gate,up} 2 x 11008x4096 (the step's largest launch)",
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": dom_ms * 1e3, "median_launch_us": dom_median_ms * 1e3,
                     "timing": "average over single dispatches of this kernel, each timed by the begin/end time stamps of its own "
                               "dispatch (HIP events handed to the launch), packed copies rotated -- the per-dispatch duration a "
                               "kernel trace reports",
                     "back_to_back_us": dom_stream_ms * 1e3, "back_to_back_GB/s": dom_bytes / dom_stream_ms / 1e6,
                     "back_to_back_note": "region of launches of this kernel alone / launches: drain and ramp-up of neighbours overlap",
                     "measured_ceiling_GB/s": ceil["50.8MB"]["per_dispatch_GB/s"],
                     "frac_of_measured_ceiling": ceil["50.8MB"]["per_dispatch_us"] / (dom_ms * 1e3),
                     "step_frac": gbs / HBM_PEAK_GBS,
                     "step_frac_of_measured_ceiling": step_ceiling_us / (ms1 * 1e3),
                     "profiled_trace_avg_us": trace_us,
                     "frac_at_profiled_trace_avg": (dom_bytes / trace_us / 1e3 / HBM_PEAK_GBS) if trace_us else None,
                     "profiled_trace_note": "average duration of this kernel in profiles/gemv_m1_llama7b_kernel_stats.txt (rocprofv3 "
                                            "--kernel-trace of this command, parsed from that file, not measured in this run): under "
                                            "the tracer every dispatch starts on an idle GPU and takes 5-8 % longer than in the "
                                            "unprofiled stream that avg_launch_us times",
                     "traffic_source": "profiles/gemv_m1_llama7b_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                                       "command, scaled by a plain copy; parsed from that file, not measured in this run"},
        "cpu_baseline": cpu,
        "legs": legs,
    }
    if gemm_roof:
        out["roofline_gemm"] = gemm_roof
    print(json.dumps(out))


if __name__ == "__main__":
    main()
