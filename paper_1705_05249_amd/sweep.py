"""On-device tile-parameter sweep (the paper's Section 3.3 tuning, scaled to one known device).

For every shape class of the five workload groups this times EVERY compiled kernel configuration
that is legal for the shape (the exhaustive "most likely" set of the paper; the table holds a few
dozen kernels, so no random sampling is needed) with a few split-K factors, keeps ALL timings
(one JSON line per (shape, kernel, split) in the output file, like the paper's database that
stores every timing, not only the best) and prints the winner per shape.  For every shape the
configuration the library selects by itself is timed as well, in the same run (kernel "auto"), so
that the regret of the selection rules in csrc/select.hip can be read off the file.  FP32 shapes with a
dimension 1 to 4 beyond a multiple of 64 are timed a second time with the fringe rows / columns taken off the
tiles (kernel name + "+fringe").  Group 4 is the
batched workload: every batched kernel on every instance size and batch count (the paper notes that
its batched routine re-used the non-batched parameters sub-optimally, Section 4.6).  An interrupted
sweep resumes: lines already in the output file are skipped.

    python -m paper_1705_05249_amd.sweep --out sweep.jsonl [--group 3] [--quick]
    python -m paper_1705_05249_amd.sweep --summary sweep.jsonl      (no GPU needed: winner, selection
                                                                                and regret per shape, as markdown)

Group 6 holds nine FP32 shapes for the problem-specific tuning experiment of the paper's Section 4.3
(Fig. 4): tune for each of nine problems, run every winner on every problem, report performance relative
to the problem's own winner.  Because the sweep times every configuration on every shape anyway, that
matrix is a pure read-out of the timing file:

    python -m paper_1705_05249_amd.sweep --cross sweep.jsonl      (no GPU needed)
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
    """seconds per call in the steady power state: after an idle spell the part needs some ten milliseconds of load
    before it holds its clock (and the first launches can be faster or slower than the steady ones), so untimed
    launches come first"""
    import torch
    from .measure import ramp
    fn()
    torch.cuda.synchronize()
    ramp(fn, 0.04)
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
        if r["shape"].startswith(prefix) and r["kernel"] != "auto":
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


def summary(path):
    """Markdown table per shape: fastest configuration, what the library selects by itself, regret."""
    times, auto = {}, {}
    for line in open(path):
        try:
            r = json.loads(line)
        except ValueError:
            continue
        if r["kernel"] == "auto":
            auto[r["shape"]] = r
        else:
            times.setdefault(r["shape"], {})[(r["kernel"], r["split_k"])] = r
    lines = ["| shape | fastest configuration | us | selected by the library | us, same pass as the others | us, automatic call | selected / fastest |",
             "|---|---|---|---|---|---|---|"]
    worst, judged = 0.0, 0
    for shape in times:
        key = min(times[shape], key=lambda c: times[shape][c]["us"])
        best = times[shape][key]
        a = auto.get(shape)
        if a is None:
            lines.append(f"| {shape} | {key[0]} split {key[1]} | {best['us']:.1f} | (not timed) | | | |")
            continue
        # the automatic call may have been timed on another box or in another power state than the forced
        # configurations; where the configuration it picked was also timed by force, that timing is the fair one
        same = times[shape].get((a["selected"], a["selected_split"]))
        own = same["us"] if same else a["us"]
        ratio = own / best["us"]
        worst = max(worst, ratio)
        judged += 1
        lines.append(f"| {shape} | {key[0]}" + (f" split {key[1]}" if key[1] > 1 else "") + f" | {best['us']:.1f} | {a['selected']}"
                     + (f" split {a['selected_split']}" if a["selected_split"] > 1 else "")
                     + (f" | {same['us']:.1f} |" if same else " | |") + f" {a['us']:.1f} | {ratio:.2f} |")
    lines.append("")
    lines.append(f"largest selected / fastest: {worst:.2f} over {judged} shapes")
    return "\n".join(lines)


def sweep_batched(log, done, quick):
    """group 4: every batched kernel on every instance size and batch count of the batched workload"""
    import torch
    from . import measure as M
    table = [t for t in G.kernel_table() if t["family"] == G.MG_FAMILY_BATCHED]
    for dtype in ("f32",) if quick else ("f32", "f16"):
        for size in (8, 16, 32, 64):
            for batch in (1000, 10000):
                name = f"c4_{dtype}_s{size}_b{batch}"
                bc = W.config4_fast(size, batch, dtype=dtype)
                t = {x: M.to_gpu(getattr(bc, x)) for x in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}
                fn = G.mg_sgemm_batched if dtype == "f32" else G.mg_hgemm_batched
                call = lambda: fn(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, t["alphas"], t["A"], t["a_off"], bc.lda, t["B"],
                                  t["b_off"], bc.ldb, t["betas"], t["C"], t["c_off"], bc.ldc, bc.batch, check=False)
                code = G.MG_F32 if dtype == "f32" else G.MG_F16
                best = None
                for k in table:
                    if k["dtype"] != code or (name, k["name"], 1) in done:
                        continue
                    G.mg_override_batched_config(k["kernel_id"])
                    if call() != 0:
                        continue                    # this kernel does not take this shape
                    secs = time_call(call)
                    rec = {"shape": name, "dtype": dtype, "m": size, "n": size, "k": size, "batch": batch, "kernel": k["name"],
                           "split_k": 1, "us": round(secs * 1e6, 2), "gflops": round(bc.flops / secs / 1e9, 1)}
                    log.write(json.dumps(rec) + "\n")
                    log.flush()
                    if best is None or secs < best[0]:
                        best = (secs, k["name"])
                G.mg_clear_override()
                if (name, "auto", 1) not in done:
                    secs = time_call(call)
                    rec = {"shape": name, "dtype": dtype, "m": size, "n": size, "k": size, "batch": batch, "kernel": "auto",
                           "split_k": 1, "selected": "(automatic)", "selected_split": 1, "us": round(secs * 1e6, 2),
                           "gflops": round(bc.flops / secs / 1e9, 1)}
                    log.write(json.dumps(rec) + "\n")
                    log.flush()
                    if best:
                        print(f"{name:28s} best {best[1]:36s} {best[0] * 1e6:10.2f} us   automatic selection {secs * 1e6:10.2f} us", flush=True)


def main():
    import torch
    ap = argparse.ArgumentParser()
    ap.add_argument("--out")
    ap.add_argument("--summary", help="timing file to summarise: winner, selection and regret per shape (no GPU needed)")
    ap.add_argument("--cross", help="timing file to read the problem-specific tuning matrix from (no GPU needed)")
    ap.add_argument("--group", type=int, action="append", help="workload group(s) 1,2,3,4,5,6 (default: all)")
    ap.add_argument("--quick", action="store_true")
    ap.add_argument("--splits", default="1,2,4,8,16")
    args = ap.parse_args()
    if args.cross:
        print(cross_matrix(args.cross))
        return 0
    if args.summary:
        print(summary(args.summary))
        return 0
    if not args.out:
        ap.error("--out or --cross is required")
    groups = set(args.group or (1, 2, 3, 4, 5, 6))
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
        if 4 in groups:
            sweep_batched(log, done, args.quick)
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
                    # the same configuration with the fringe rows / columns left to the extra work-groups
                    if dtype != "f32" or (name, t["name"] + "+fringe", split) in done:
                        continue
                    G.mg_override_fringe(G.MG_FRINGE_ON)
                    ok = G.lib().mg_query_selected(code, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta, 16, ctypes.byref(cfg)) == 0
                    if ok and cfg.fringe != 0:
                        secs = time_call(lambda: fn(layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cd, ldc, ws))
                        rec = {"shape": name, "dtype": dtype, "m": m, "n": n, "k": k, "kernel": t["name"] + "+fringe",
                               "split_k": split, "us": round(secs * 1e6, 2), "gflops": round(flops / secs / 1e9, 1)}
                        log.write(json.dumps(rec) + "\n")
                        log.flush()
                        if secs < best[name][0]:
                            best[name] = (secs, t["name"] + "+fringe", split)
                    G.mg_override_fringe(G.MG_FRINGE_AUTO)
            G.mg_clear_override()
            sel = G.mg_query_selected(code, layout, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta, 16)
            if (name, "auto", 1) not in done:
                # what the library does by itself, with the workspace its preferred route asks for
                need = G.mg_gemm_workspace_bytes(code, layout, ta, tb, m, n, k, lda, ldb, ldc)
                auto_ws = ws[:max(need, 256)] if need else None
                secs = time_call(lambda: fn(layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, Cd, ldc, auto_ws))
                rec = {"shape": name, "dtype": dtype, "m": m, "n": n, "k": k, "kernel": "auto", "split_k": 1,
                       "selected": sel["name"] + ("+fringe" if sel["fringe"] else ""), "selected_split": sel["split_k"],
                       "us": round(secs * 1e6, 2), "gflops": round(flops / secs / 1e9, 1)}
                log.write(json.dumps(rec) + "\n")
                log.flush()
            if name in best:
                secs, kname, split = best[name]
                print(f"{name:28s} best {kname:36s} split={split:<3d} {secs * 1e6:10.1f} us {flops / secs / 1e12:9.2f} TFLOPS"
                      f"   (auto-selected: {sel['name']} split={sel['split_k']})", flush=True)
    G.mg_clear_override()


if __name__ == "__main__":
    sys.exit(main())
