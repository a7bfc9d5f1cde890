"""On-device tile-parameter sweep (the paper's Section 3.3 tuning, scaled to one known device).

For every shape class of the five workload groups this times EVERY compiled kernel configuration
that is legal for the shape (the exhaustive "most likely" set of the paper; the table holds a few
dozen kernels, so no random sampling is needed) with a few split-K factors, keeps ALL timings
(one JSON line per (shape, kernel, split) in the output file, like the paper's database that
stores every timing, not only the best) and prints the winner per shape.  The selection table in
csrc/select.hip is written from these winners.  An interrupted sweep resumes: lines already in
the output file are skipped.

    python -m paper_1705_05249_amd.sweep --out gpurun_out/sweep.jsonl [--group 3] [--quick]

Group 6 holds nine FP32 shapes for the problem-specific tuning experiment of the paper's Section 4.3
(Fig. 4): tune for each of nine problems, run every winner on every problem, report performance relative
to the problem's own winner.  Because the sweep times every configuration on every shape anyway, that
matrix is a pure read-out of the timing file:

    python -m paper_1705_05249_amd.sweep --cross gpurun_out/sweep.jsonl      (no GPU needed)
"""
import argparse
import ctypes
import json
import os
import sys

from . import gemm as G
from . import workloads as W


def shapes(groups, quick):
    """(name, dtype, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta)"""
    out = []
    C, R, N, T = W.COL_MAJOR, W.ROW_MAJOR, W.NO_TRANS, W.TRANS

    def tight(layout, ta, tb, m, n, k):
        return W.tight_ld(layout, ta, m, k), W.tight_ld(layout, tb, k, n), W.tight_ld(layout, N, m, n)

    if 1 in groups:
        out.append(("c1_256", "f32", C, N, N, 256, 256, 256, 256, 256, 256, 1.5, 0.5))
    if 2 in groups:
        for size in ((1024, 4096) if quick else W.CONFIG2_SIZES):
            for ta, tb in ((N, N), (N, T), (T, N), (T, T)):
                for beta in W.CONFIG2_BETAS:
                    out.append((f"c2_{size}_{'NT'[ta == T]}{'NT'[tb == T]}_b{beta}", "f32", C, ta, tb, size, size, size,
                                *tight(C, ta, tb, size, size, size), 1.0, beta))
    if 3 in groups:
        for m, n, k in W.CONFIG3_SHAPES:
            out.append((f"c3_{m}x{n}x{k}", "f16", C, N, N, m, n, k, *tight(C, N, N, m, n, k), 1.0, 0.0))
    if 5 in groups:
        for m, n, k in W.CONFIG5_SHAPES:
            out.append((f"c5_{m}x{n}x{k}", "f32", C, T, N, m, n, k, W.padded_ld(k), W.padded_ld(k), W.padded_ld(m),
                        1.0, 1.0))
    if 6 in groups:
        for m, n, k in CROSS_SHAPES:
            out.append((f"x_{m}x{n}x{k}", "f32", C, N, N, m, n, k, *tight(C, N, N, m, n, k), 1.0, 0.0))
    return out


# problem-specific tuning experiment: squares from launch-bound to compute-bound, short K, skinny, ragged
CROSS_SHAPES = ((256, 256, 256), (512, 512, 512), (1024, 1024, 1024), (2048, 2048, 2048), (4096, 4096, 4096),
                (4096, 4096, 64), (64, 4096, 4096), (4096, 64, 4096), (1000, 1001, 999))


def graph_time(fn, per_graph=20, replays=10):
    """seconds per call from replays of a HIP graph of `per_graph` calls (calls shorter than the host's launch
    cost cannot be timed back to back from Python)"""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(per_graph):
            fn()
    graph.replay()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(replays):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3 / (replays * per_graph)


def time_call(fn, min_seconds=2e-3, max_reps=200):
    import torch
    fn()
    torch.cuda.synchronize()
    reps = 3
    while True:
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            fn()
        stop.record()
        torch.cuda.synchronize()
        total = start.elapsed_time(stop) * 1e-3
        if total >= min_seconds or reps >= max_reps:
            if total / reps < 40e-6:
                return min(total / reps, graph_time(fn))
            return total / reps
        reps = min(max_reps, max(reps * 2, int(reps * min_seconds / max(total, 1e-7)) + 1))


def cross_matrix(path, prefix="x_"):
    """Markdown table: rows = problems, columns = the configuration tuned for each problem; entry = the row
    problem's throughput with that configuration relative to its own best (the diagonal is 100).  A
    configuration is (tile kernel, split-K factor); where a problem needs the bounds-checked flavour of a tile
    kernel (or may use the unchecked one) that flavour stands in, the tile parameters being the same."""
    times = {}
    for line in open(path):
        try:
            r = json.loads(line)
        except ValueError:
            continue
        if r["shape"].startswith(prefix):
            times.setdefault(r["shape"], {})[(r["kernel"], r["split_k"])] = r["us"]
    order = [f"{prefix}{m}x{n}x{k}" for m, n, k in CROSS_SHAPES if f"{prefix}{m}x{n}x{k}" in times]
    winners = {shape: min(times[shape], key=times[shape].get) for shape in order}

    def flavours(kernel):
        base = kernel[:-5] if kernel.endswith("_edge") else kernel
        return (kernel, base + "_edge", base)

    lines = ["| problem \\ tuned for | " + " | ".join(s[len(prefix):] for s in order) + " | best configuration | GFLOPS |",
             "|---|" + "---|" * (len(order) + 2)]
    for shape in order:
        best_us = times[shape][winners[shape]]
        cells = []
        for other in order:
            kernel, split = winners[other]
            us = next((times[shape][(f, split)] for f in flavours(kernel) if (f, split) in times[shape]), None)
            cells.append("-" if us is None else f"{100.0 * best_us / us:.0f}")
        m, n, k = (int(x) for x in shape[len(prefix):].split("x"))
        kernel, split = winners[shape]
        lines.append(f"| {shape[len(prefix):]} | " + " | ".join(cells) + f" | {kernel} split {split} | "
                     f"{2.0 * m * n * k / best_us / 1e3:.0f} |")
    return "\n".join(lines)


def main():
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--out")
    ap.add_argument("--cross", help="timing file to read the problem-specific tuning matrix from (no GPU needed)")
    ap.add_argument("--group", type=int, action="append", help="workload group(s) 1,2,3,5,6 (default: all)")
    ap.add_argument("--quick", action="store_true")
    ap.add_argument("--splits", default="1,2,4,8,16")
    args = ap.parse_args()
    if args.cross:
        print(cross_matrix(args.cross))
        return 0
    if not args.out:
        ap.error("--out or --cross is required")
    groups = set(args.group or (1, 2, 3, 5, 6))
    splits = [int(x) for x in args.splits.split(",")]
    done = set()
    if os.path.exists(args.out):
        for line in open(args.out):
            try:
                r = json.loads(line)
                done.add((r["shape"], r["kernel"], r["split_k"]))
            except ValueError:
                pass
    table = G.kernel_table()
    ws = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    best = {}
    with open(args.out, "a") as log:
        for (name, dtype, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta) in shapes(groups, args.quick):
            code = G.MG_F32 if dtype == "f32" else G.MG_F16
            tdt = torch.float32 if dtype == "f32" else torch.float16
            fn = G.mg_sgemm if dtype == "f32" else G.mg_hgemm
            sa = W.storage_len(layout, ta, m, k, lda)
            sb = W.storage_len(layout, tb, k, n, ldb)
            sc = W.storage_len(layout, W.NO_TRANS, m, n, ldc)
            A = (torch.rand(sa, device="cuda") - 0.5).to(tdt)
            B = (torch.rand(sb, device="cuda") - 0.5).to(tdt)
            Cd = torch.zeros(sc, device="cuda", dtype=tdt)
            flops = 2.0 * m * n * k
            for t in table:
                if t["dtype"] != code or t["family"] in (G.MG_FAMILY_BATCHED, G.MG_FAMILY_SCALE):
                    continue
                if t["family"] == G.MG_FAMILY_DIRECT and flops > 2e10:
                    continue            # the direct kernel is the small-problem fallback
                for split in splits:
                    if (name, t["name"], split) in done:
                        continue
                    if G.mg_override_config(t["kernel_id"], split, check=False) != 0:
                        continue
                    cfg = G.mg_config()
                    if G.lib().mg_query_selected(code, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta, 16,
                                                 ctypes.byref(cfg)) != 0:
                        continue
                    need = G.mg_gemm_workspace_bytes(code, layout, ta, tb, m, n, k, lda, ldb, ldc)
                    if need > ws.numel():
                        continue
                    secs = time_call(lambda: fn(layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cd, ldc, ws))
                    rec = {"shape": name, "dtype": dtype, "m": m, "n": n, "k": k, "kernel": t["name"], "split_k": split,
                           "us": round(secs * 1e6, 2), "gflops": round(flops / secs / 1e9, 1)}
                    log.write(json.dumps(rec) + "\n")
                    log.flush()
                    if name not in best or secs < best[name][0]:
                        best[name] = (secs, t["name"], split)
            G.mg_clear_override()
            if name in best:
                secs, kname, split = best[name]
                sel = G.mg_query_selected(code, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta, 16)
                print(f"{name:28s} best {kname:36s} split={split:<3d} {secs * 1e6:10.1f} us {flops / secs / 1e12:9.2f} TFLOPS"
                      f"   (auto-selected: {sel['name']} split={sel['split_k']})", flush=True)
    G.mg_clear_override()


if __name__ == "__main__":
    sys.exit(main())
