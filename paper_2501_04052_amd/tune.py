"""Offline launch-shape tuner (the counterpart of the paper's auto-tuning strategy, Sec. 4.3 / App. E).

For every problem of the shape list -- the projections of Llama-7B- and 70B-shaped decoder layers, as
single matrices and as the fused {q,k,v} / {gate,up} groups, at the batch sizes of the decode regime --
every launch shape of the problem's kernel family (include/razer_tune.h) is forced in turn through
razer_tune_force and timed on the GPU: HIP events around a region of back-to-back calls that rotate
through enough copies of the packed weights to defeat the last-level cache.  The fastest shape goes
into the table, unless the heuristic's own shape is within `--margin` of it.

    python -m paper_2501_04052_amd.tune            # sweep, print the table
    python -m paper_2501_04052_amd.tune --write    # ... and write csrc/razer_tuned.inc (rebuild afterwards)

Timing only: packed bytes are random (kernel speed does not depend on the values).
"""
import argparse
import json
import os
import sys
import time

_PKG = os.path.dirname(os.path.abspath(__file__))
TABLE_PATH = os.path.join(_PKG, "csrc", "razer_tuned.inc")
LLC_BYTES = 256 << 20

FAMILY_NAMES = {0: "RAZER_TUNE_GEMV", 1: "RAZER_TUNE_GEMV_QUAD", 2: "RAZER_TUNE_SMALL_BATCH", 3: "RAZER_TUNE_GEMM_SLICES"}


def candidates(family, m, k):
    """Launch shapes of a family that the kernels are built for, for this m and k."""
    if family == 0:
        waves = -(-k // 2048)
        return [(2, 1), (4, 1), (8, 1)] + ([(2, 2)] if waves <= 8 else [])
    if family == 1:
        return [(4,), (8,)] if k <= 16384 else [(4,)]
    if family == 2:
        sliced = [(0, 4, 1), (0, 4, 2), (0, 4, 4)] + ([(0, 8, 1), (0, 8, 2)] if m <= 16 else [])
        inside = [(1, 1, 1), (1, 1, 2), (1, 1, 3), (1, 1, 4), (1, 2, 1), (1, 2, 2), (1, 2, 3), (1, 2, 4), (1, 2, 8)] if m <= 16 else []
        return sliced + inside
    kt = -(-k // 64)
    return [(s,) for s in (1, 2, 3, 4, 6, 8, 12, 16) if s <= kt]


def family_of(m, k, block=16):
    if m <= 1 or (m <= 4 and k > 32768):
        return 0 if k <= 32768 else None
    if m <= 4:
        return 1
    if m <= 32:
        return 2
    if m <= 128:
        return 3
    return None


def problems():
    """(m, rows of the matrices of one call, k)."""
    from .synth import LLAMA_7B_LAYER, LLAMA_70B_LAYER
    out = []
    for layer in (LLAMA_7B_LAYER, LLAMA_70B_LAYER):
        rows = {name: n for name, n, _ in layer}
        ks = {name: k for name, _, k in layer}
        calls = [((rows["q"], rows["k"], rows["v"]), ks["q"]), ((rows["o"],), ks["o"]),
                 ((rows["gate"], rows["up"]), ks["gate"]), ((rows["down"],), ks["down"]),
                 ((rows["q"],), ks["q"]), ((rows["gate"],), ks["gate"])]
        if rows["k"] != rows["q"]:
            calls.append(((rows["k"],), ks["k"]))
        for ns, k in calls:
            for m in (1, 2, 3, 4, 5, 8, 12, 16, 24, 32, 64, 128):
                out.append((m, ns, k))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--write", action="store_true", help="write csrc/razer_tuned.inc")
    ap.add_argument("--margin", type=float, default=0.04, help="keep the heuristic unless a shape is this much faster")
    ap.add_argument("--launches", type=int, default=60)
    ap.add_argument("--out", default=None, help="also write the sweep as JSON lines to this file")
    ap.add_argument("--only-m", type=int, nargs="*", default=None)
    args = ap.parse_args()
    import torch
    from . import binding as rz
    rz.load_library()
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    stream = torch.cuda.current_stream().cuda_stream
    entries, log = [], []
    pool_cache = {}

    def packed_copies(ns, k):
        key = (ns, k)
        if key not in pool_cache:
            pool_cache.clear()
            torch.cuda.empty_cache()
            per_copy = sum(n * k * 9 // 16 for n in ns)
            copies = max(2, min(40, -(-2 * LLC_BYTES // per_copy)))
            sets = []
            for _ in range(copies):
                sets.append([rz.RazerTensor(
                    torch.randint(0, 256, (n, k // 2), generator=gen, device="cuda", dtype=torch.uint8),
                    torch.randint(0, 256, (n, k // 16), generator=gen, device="cuda", dtype=torch.uint8),
                    torch.tensor([1e-3], device="cuda"), n, k, rz.WEIGHT, (5.0, 8.0)) for n in ns])
            pool_cache[key] = sets
        return pool_cache[key]

    def time_calls(calls, launches):
        n = len(calls)
        for i in range(10):
            calls[i % n](stream)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(launches):
                calls[i % n](stream)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e3 / launches
            best = t if best is None else min(best, t)
        return best

    t_start = time.time()
    for m, ns, k in problems():
        if args.only_m and m not in args.only_m:
            continue
        fam = family_of(m, k)
        if fam is None:
            continue
        sets = packed_copies(ns, k)
        a = torch.randn((m, k), generator=gen, device="cuda").to(torch.bfloat16)
        outs = [torch.empty((m, n), dtype=torch.bfloat16, device="cuda") for n in ns]

        def build():
            # (prepared after forcing: the workspace is sized for the forced shape)
            if len(ns) == 1:
                return [rz.prepare_linear(s[0], a, outs[0]) for s in sets]
            return [rz.prepare_linear_grouped(s, a, outs) for s in sets]
        rz.razer_tune_force(fam, None)
        src, _ = rz.razer_tune_lookup(fam, m, sum(ns), k)
        rz.razer_tune_force(fam, (-1, -1, -1, -1))            # an unbuilt shape: the heuristic, whatever the table says
        t_default = time_calls(build(), args.launches)
        results = []
        for shape in candidates(fam, m, k):
            rz.razer_tune_force(fam, shape)
            results.append((time_calls(build(), args.launches), shape))
        rz.razer_tune_force(fam, (-1, -1, -1, -1))            # the heuristic once more: the smaller of the two readings
        t_default = min(t_default, time_calls(build(), args.launches))
        rz.razer_tune_force(fam, None)
        t_best, best = min(results)
        rec = {"m": m, "rows": list(ns), "k": k, "family": fam, "default_us": t_default,
               "best_us": t_best, "best": list(best), "all": [[list(s), t] for t, s in results]}
        log.append(rec)
        keep = t_best < t_default * (1.0 - args.margin)
        print("m=%-4d rows=%-22s k=%-6d %-24s default %7.2f us  best %-12s %7.2f us %s"
              % (m, "+".join(map(str, ns)), k, FAMILY_NAMES[fam], t_default, best, t_best, "<- table" if keep else ""),
              flush=True)
        if keep:
            entries.append((fam, m, sum(ns), k, tuple(best) + (0,) * (4 - len(best)), t_default, t_best))
    print("# sweep took %.0f s, %d table entries" % (time.time() - t_start, len(entries)), flush=True)
    # one entry per key (a single matrix and a group can share (m, rows, k): the group wins, it is listed first)
    seen, lines = set(), []
    for fam, m, rows, k, p, t0, t1 in entries:
        if (fam, m, rows, k) in seen:
            continue
        seen.add((fam, m, rows, k))
        lines.append("    {%d, %d, %d, %d, {%d, %d, %d, %d}},   // %s: %.1f -> %.1f us"
                     % (fam, m, rows, k, p[0], p[1], p[2], p[3], FAMILY_NAMES[fam], t0, t1))
    header = ("// Launch shapes measured on an MI355X by `python -m paper_2501_04052_amd.tune --write`\n"
              "// {family, m, rows (summed over a group), cols, {p0, p1, p2, p3}}; families and parameters: include/razer_tune.h\n")
    text = header + "\n".join(lines) + ("\n" if lines else "")
    print(text)
    if args.write:
        with open(TABLE_PATH, "w") as f:
            f.write(text)
    if args.out:
        with open(args.out, "w") as f:
            for rec in log:
                f.write(json.dumps(rec) + "\n")
            f.write("#TABLE\n" + text)


if __name__ == "__main__":
    main()
