"""Benchmark of the GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only GROUP] [--no-cpu-baseline]

One "step" is one mg_hgemm call on the headline workload: FP16 storage / FP32 accumulation, column-major,
op(A)=A, op(B)=B, m=n=k=4096, alpha=1, beta=0, entries N(0, K^-1/2) rounded to FP16 (seeded, synthetic).  Inputs are
resident in HBM before the timed region; W warm-up steps, then exactly K steps between two device
synchronisations.  Prints ONE JSON line: GFLOPS = 2mnk/t, the MFMA roofline of the kernel, the CPU oracle timed on
a bounded sample of the same workload (cpu_baseline), and under "workloads" every other workload of the five
configurations (each with the roofline that bounds it), the cold (HBM-real) variants of the small ones, the
launch floor, the rate of the matrix pipes alone, where the headline kernel's time goes ("accounting"), and the
paper's own figures for context ("paper_context").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2500.0, "f32": 157.3}     # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
GROUPS = ("hgemm", "probes", "config1", "config2", "sgemm", "config3", "config4", "batched", "config5", "conv", "gemv",
          "level3", "copy")

# What the paper itself reports for this path (its OpenCL devices of 2012-2017; context, not targets).
PAPER_CONTEXT = [
    "HGEMM: 'over 200 GFLOPS' on Intel Skylake ULT GT2 (peak 384 GFLOPS FP32, 30 GB/s), FP16 compute (Section 4.4)",
    "HGEMM about 2x SGEMM on Skylake ULT GT2 and ARM Mali T628 (Section 4.4)",
    "batched GEMM 'up to an order of magnitude' faster than a loop of small GEMMs on GTX 750Ti and Skylake ULT GT2 (Section 4.6)",
    "generic batched up to 2x slower than strided batched on GTX 750Ti: per-instance offsets and scalars (Section 4.6)",
    "problem-specific tuning gains up to 2x on Radeon M370X, 9 sizes x 9 parameter sets (Section 4.3)",
    "device peaks of the paper's Table 2 (GFLOPS FP32 - GB/s): GTX 750Ti 1305-88, Titan X Pascal 10974-480, HD7970 3789-264, "
    "M370X 1024-72, Skylake ULT GT2 384-30, Mali T628 38-15",
]


def measured_traffic():
    """HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, as written to profiles/traffic.json
    together with the commit they were measured at (never measured in this run: null where the file has no entry)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {"measured_at_commit": None, "bytes_per_launch": {}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-probes", action="store_true", help="skip the measuring aids (profiling runs of a single kernel)")
    ap.add_argument("--only", default=None, help=" | ".join(GROUPS) + ": run a single group (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if args.only is not None and args.only not in GROUPS:
        sys.exit(f"--only takes one of {GROUPS}")

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    from paper_1705_05249_amd import gemm as G, measure as M, workloads as W
    G.lib()
    G.mg_clear_override()
    steps, warmup = args.steps, args.warmup
    extra = []
    traffic = measured_traffic()

    def want(*groups):
        return args.only is None or args.only in groups

    def roofline(bound, work, seconds, peak, key):
        """work: algorithmic flops (bound mfma) or bytes (bound hbm) of one launch"""
        if bound == "mfma":
            achieved, unit = work / seconds / 1e12, "TFLOP/s"
        else:
            achieved, unit = work / seconds / 1e9, "GB/s"
        return {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit, "frac": round(achieved / peak, 4),
                "traffic": traffic["bytes_per_launch"].get(key)}

    def gemm_setup(case):
        fn = G.mg_sgemm if case.dtype == "f32" else G.mg_hgemm
        code = G.MG_F32 if case.dtype == "f32" else G.MG_F16
        A, B, C = M.to_gpu(case.A), M.to_gpu(case.B), M.to_gpu(case.C)
        need = G.mg_gemm_workspace_bytes(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb,
                                         case.ldc)
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None
        sel = G.mg_query_selected(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb, case.ldc,
                                  case.alpha, case.beta)

        def call_on(a, b, c):
            return lambda: fn(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, a, case.lda, b, case.ldb,
                              case.beta, c, case.ldc, ws)

        return A, B, C, sel, call_on

    def gemm_entry(label, case, bound, key=None, small=False, cold=False, reps=None):
        """one GEMM workload: events around back-to-back calls, or (small) graph replays; cold: also the time per call
        when the operands come from HBM (a cycle through copies that together exceed the last-level cache four times)"""
        A, B, C, sel, call_on = gemm_setup(case)
        entry = {"workload": label, "kernel": sel["name"] + (f" split {sel['split_k']}" if sel["split_k"] > 1 else "")
                 + (f" + fringe of {sel['fringe'] // 16} row(s), {sel['fringe'] % 16} column(s)" if sel["fringe"] else "")}
        if small:
            dev_graph, dev_eager = M.graph_timed(call_on(A, B, C), C, steps, warmup)
            entry["ms_graph_replays"] = round(dev_graph * 1e3, 5)
            entry["ms_eager_launches"] = round(dev_eager * 1e3, 5)
            # calls the host can issue faster than they run are back to back either way; a replay adds its own start-up
            dev = min(dev_graph, dev_eager)
        else:
            M.ramp(call_on(A, B, C))
            dev, _ = M.timed(call_on(A, B, C), reps or max(5, steps // 5), max(1, warmup // 4))
        entry["gflops"] = round(case.flops / dev / 1e9, 1)
        entry["ms"] = round(dev * 1e3, 5)
        peak = PEAK_TFLOPS[case.dtype] if bound == "mfma" else PEAK_HBM_GBS
        work = case.flops if bound == "mfma" else case.algorithmic_bytes
        entry["roofline"] = roofline(bound, work, dev, peak, key or label)
        nbytes = A.numel() * A.element_size() + B.numel() * B.element_size() + C.numel() * C.element_size()
        if nbytes < M.LAST_LEVEL_CACHE_BYTES:
            entry["note"] = (f"{nbytes / 1e6:.1f} MB of operands: repeated calls are served by the 256 MB last-level cache"
                             + ("; the faster of eager launches and replays of a HIP graph of 20 launches" if small else ""))
        if cold:
            copies = []

            def make_call(i):
                copies.append((A.clone(), B.clone(), C.clone()))
                return call_on(*copies[-1])

            dev_cold, sets = M.cold_timed(make_call, nbytes)
            entry["cold"] = {"ms": round(dev_cold * 1e3, 5), "gflops": round(case.flops / dev_cold / 1e9, 1), "sets": sets,
                             "roofline": roofline(bound, work, dev_cold, peak, None),
                             "note": f"graph replay of one cycle over {sets} distinct copies of A, B, C ({sets * nbytes / 2**30:.2f} GiB)"}
            del copies
        extra.append(entry)
        return entry

    if args.only == "copy":
        # calibration for the FETCH_SIZE / WRITE_SIZE counters: a plain device copy of known size
        # (1 GiB read + 1 GiB written, far beyond the 256 MB last-level cache)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "launches": 3}))
        return

    # ---- headline: HGEMM 4096^3 ------------------------------------------------------------------
    head = None
    if want("hgemm"):
        case = W.config3(4)
        A, B, C, sel, call_on = gemm_setup(case)
        M.ramp(call_on(A, B, C))            # clock ramp after the idle spell of input generation; then W warm-up steps, K timed
        dev, wall = M.timed(call_on(A, B, C), steps, warmup)
        head = {"case": case, "dev": dev, "wall": wall, "sel": sel, "fastest": M.fastest_single(call_on(A, B, C))}
        cpu = None
        if not args.no_cpu_baseline:
            from oracle import gemm_oracle
            # bounded sample of the same workload: complete rows/columns + scattered entries (about 10-30 s)
            rows, cols = W.sample_entries(case.m, case.n, seed=4096, rows=256, cols=256, scattered=8192)
            t0 = time.perf_counter()
            c_ref, d_ref = gemm_oracle.gemm_entries("f16", case.layout, case.ta, case.tb, case.m, case.n, case.k,
                                                    case.alpha, case.A, case.lda, case.B, case.ldb, case.beta,
                                                    case.C, case.ldc, rows, cols)
            t_cpu = time.perf_counter() - t0
            got = W.unpack(C.cpu().numpy(), case.layout, case.m, case.n, case.ldc)[rows, cols]
            err = M.rel_error(got, c_ref, d_ref)
            assert err <= 2e-3, f"benchmark output fails parity: {err}"
            cpu = {"value": round(2.0 * case.k * rows.size / t_cpu / 1e9, 3), "unit": "GFLOPS",
                   "cores": gemm_oracle.threads(), "kind": "oracle",
                   "sample": f"{rows.size} of {case.m * case.n} output entries (256 full rows, 256 full columns, "
                             f"8192 scattered), each a full k={case.k} FP64 dot product; {t_cpu:.1f} s",
                   "max_rel_err_gpu_vs_oracle": float(f"{err:.3e}")}
        head["cpu"] = cpu
        head["buffers"] = (A, B, C)

    # ---- what the fractions are judged against: launch floor, the matrix pipes alone, where the kernel's time goes
    probes = {}
    if want("probes", "hgemm") and not args.no_probes:
        flag = torch.zeros(1, dtype=torch.float32, device="cuda")
        floor_graph, floor_eager = M.graph_timed(lambda: G.mg_probe_empty_launch(), flag, steps, warmup)
        probes["launch_floor"] = {"us_back_to_back_in_a_graph": round(floor_graph * 1e6, 3),
                                  "us_eager_from_python": round(floor_eager * 1e6, 3),
                                  "note": "one empty kernel of one wavefront per launch"}
        rounds = 128                      # 2 * 16*16*32 * 32 * rounds * 2048 wavefronts = the flops of 4096^3
        flops = 2.0 * 16 * 16 * 32 * 32 * rounds * 2048
        M.ramp(lambda: G.mg_probe_mfma_only(rounds, flag), 0.02)
        dev, _ = M.timed(lambda: G.mg_probe_mfma_only(rounds, flag), max(5, steps // 4), max(1, warmup // 4))
        probes["mfma_pipes_alone"] = {"ms": round(dev * 1e3, 5), "tflops": round(flops / dev / 1e12, 1),
                                      "frac_of_peak": round(flops / dev / 1e12 / PEAK_TFLOPS["f16"], 4),
                                      "note": "v_mfma_f32_16x16x32_f16 only, register operands that change with every "
                                              "instruction, two wavefronts per SIMD, the flops of one 4096^3 product: "
                                              "what the part sustains at the clock it holds under this load"}
        if head is not None:
            A, B, C = head["buffers"]
            case = head["case"]
            per = 12
            groups = (case.m // 256) * (case.n // 256)
            stamps = [torch.zeros(groups * 8 * per, dtype=torch.int64, device="cuda") for _ in range(3)]
            for _ in range(3):
                G.mg_probe_hgemm_stamps(case.m, case.n, case.k, A, case.lda, B, case.ldb, C, case.ldc, stamps[0])
            for s in stamps:               # three launches back to back
                G.mg_probe_hgemm_stamps(case.m, case.n, case.k, A, case.lda, B, case.ldb, C, case.ldc, s)
            torch.cuda.synchronize()
            h = [s.cpu().numpy().reshape(groups * 8, per).astype(np.float64) for s in stamps]
            mid = h[1]
            ktiles = case.k // 64
            clock = (mid[:, 0] + mid[:, 1]) / mid[:, 2] * 0.1                  # GHz per wavefront
            by_die = {}
            for die in sorted(set(mid[:, 10].astype(int))):
                rows_ = mid[mid[:, 10] == die]
                by_die[str(die)] = {"clock_ghz": round(float(((rows_[:, 0] + rows_[:, 1]) / rows_[:, 2]).mean() * 0.1), 3),
                                    "us": round(float(rows_[:, 2].mean() * 0.01), 2)}
            span = lambda x: (x[:, 8].min(), x[:, 8].max(), x[:, 9].min(), x[:, 9].max())
            b0, b1, e0, e1 = span(h[1])
            _, _, _, prev_end = span(h[0])
            nb0, _, _, _ = span(h[2])
            loop = mid[:, 0] - mid[:, 7]
            probes["accounting_hgemm_4096"] = {
                "kernel": "the selected kernel built with cycle stamps (mg_probe_hgemm_stamps), second of three back-to-back launches",
                "us_launch_period": round(float(nb0 - b0) * 0.01, 2),
                "us_gap_last_wavefront_end_to_next_first_start": round(float(b0 - prev_end) * 0.01, 2),
                "us_first_to_last_wavefront_start": round(float(b1 - b0) * 0.01, 2),
                "us_first_to_last_wavefront_end": round(float(e1 - e0) * 0.01, 2),
                "us_wavefront_mean": round(float(mid[:, 2].mean()) * 0.01, 2),
                "us_wavefront_slowest_die": max(v["us"] for v in by_die.values()),
                "clock_ghz_mean": round(float(clock.mean()), 3),
                "per_die": by_die,
                "ticks_to_first_tile": round(float(mid[:, 7].mean())),
                "ticks_k_loop_per_tile": round(float(loop.mean()) / ktiles, 1),
                "ticks_mfma_run_per_tile": round(float(mid[:, 5].mean()) / ktiles, 1),
                "ticks_lds_reads_per_tile": round(float(mid[:, 3].mean()) / ktiles, 1),
                "ticks_barrier_waits_per_tile": round(float((mid[:, 4] + mid[:, 6]).mean()) / ktiles, 1),
                "ticks_epilogue": round(float(mid[:, 1].mean())),
                "ideal_ticks_per_tile": 2048,
                "note": "ticks of the shader clock; a K-tile is 2 x 64 MFMAs of 16 cycles per SIMD = 2048 cycles at best; "
                        "the kernel ends with its slowest die; at the mean clock and 2048 ticks per tile the K loops "
                        f"alone take {ktiles * 2048 / float(clock.mean()) * 1e-3:.1f} us",
            }
            # the kernels this one replaced, by override, in the same process (boxes differ by up to 10 %)
            call = gemm_setup(case)[4](A, B, C)
            beside = {}
            for name in ("hpp16_256x256x64_w2x4_mk", "hdma16_256x256x64_w2x4_mk", "hdma_256x256x64_w2x2_mk", "hmfma_256x256x64_w2x2_mk"):
                try:
                    G.mg_override_config(G.kernel_id(name), 1)
                except KeyError:
                    continue
                M.ramp(call, 0.02)
                dev, _ = M.timed(call, max(5, steps // 2), max(1, warmup // 2))
                beside[name] = round(dev * 1e3, 5)
                G.mg_clear_override()
            probes["hgemm_4096_ms_by_kernel"] = beside
            # the same launch on other data: what the part draws, and with it the clock it holds, depends on how many
            # bits toggle in the matrix pipes
            by_data = {}
            for tag, make in (("zeros", lambda t: torch.zeros_like(t)), ("ones", lambda t: torch.ones_like(t)),
                              ("integers in [-2, 2]", lambda t: torch.randint(-2, 3, t.shape, device="cuda").to(t.dtype)),
                              ("the workload's N(0, 1/sqrt(k))", lambda t: t)):
                a2, b2 = make(A), make(B)
                M.ramp(gemm_setup(case)[4](a2, b2, C), 0.02)
                dev, _ = M.timed(gemm_setup(case)[4](a2, b2, C), max(5, steps // 2), max(1, warmup // 2))
                by_data[tag] = {"ms": round(dev * 1e3, 5), "frac_of_peak": round(case.flops / dev / 1e12 / PEAK_TFLOPS["f16"], 4)}
            probes["hgemm_4096_by_operand_data"] = by_data
            head.pop("buffers")

    # ---- configuration 1: 256^3 (launch- and latency-bound) -----------------------------------------
    if want("config1"):
        gemm_entry("sgemm_f32_256x256x256_colmajor_NN_alpha1.5_beta0.5", W.config1(integer=False), "mfma", small=True, cold=True)

    # ---- configuration 2: FP32 squares, the four operand orders, both layouts -----------------------
    if want("config2", "sgemm"):
        N, T, CM, RM = W.NO_TRANS, W.TRANS, W.COL_MAJOR, W.ROW_MAJOR
        sizes = (4096,) if args.only == "sgemm" else W.CONFIG2_SIZES
        for size in sizes:
            logical = W.config2_logical(size)
            variants = [(CM, N, N, 0.0)]
            if size == 4096 and args.only != "sgemm":
                variants += [(CM, T, N, 0.7), (CM, N, T, 0.7), (CM, T, T, 0.7), (RM, N, N, 0.7)]
            for layout, ta, tb, beta in variants:
                case = W.config2_variant(size, layout, ta, tb, beta, logical)
                tag = ("rowmajor" if layout == RM else "colmajor") + "_" + ("T" if ta == T else "N") + ("T" if tb == T else "N")
                label = f"sgemm_f32_{size}x{size}x{size}_{tag}_beta{beta:g}"
                gemm_entry(label, case, "mfma", key="sgemm_f32_4096x4096x4096_colmajor_NN_beta0" if label.endswith("4096_colmajor_NN_beta0") else None,
                           small=size <= 1024, reps=3 if size >= 8192 else None)
            del logical

    # ---- configuration 3: the FP16 convolution-as-GEMM shapes alone ----------------------------------
    if want("config3"):
        for index in range(4):
            case = W.config3(index)
            gemm_entry(f"hgemm_f16_{case.m}x{case.n}x{case.k}_colmajor_NN_beta0", case, "hbm", small=True, cold=True)
            extra[-1]["roofline_mfma"] = {"bound": "mfma", "achieved": round(extra[-1]["gflops"] / 1e3, 2), "peak": PEAK_TFLOPS["f16"],
                                          "unit": "TFLOP/s", "frac": round(extra[-1]["gflops"] / 1e3 / PEAK_TFLOPS["f16"], 4)}

        # beyond the workload list: the same kernels where the fixed costs of a launch are 1 % instead of 10 %, and the
        # operand order with both matrices along k
        gemm_entry("hgemm_f16_8192x8192x8192_colmajor_NN_beta0 (not in the paper's list: amortised fixed costs)",
                   W.hgemm_case(8192, 8192, 8192, case=8), "mfma", reps=5)
        gemm_entry("hgemm_f16_4096x4096x4096_colmajor_TN_beta0 (not in the paper's list: both operands along k)",
                   W.hgemm_case(4096, 4096, 4096, case=9, ta=W.TRANS), "mfma", reps=max(5, steps // 5))

    # ---- configuration 4: batched GEMM -------------------------------------------------------------
    if want("config4", "batched"):
        def batched_entry(label, bc, strided=False, cold_batch=None):
            half = bc.dtype == "f16"
            t = {name: M.to_gpu(getattr(bc, name)) for name in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}
            stride = int(bc.a_off[1] - bc.a_off[0])
            generic_fn = G.mg_hgemm_batched if half else G.mg_sgemm_batched
            strided_fn = G.mg_hgemm_strided_batched if half else G.mg_sgemm_strided_batched
            if strided:
                call = lambda: strided_fn(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, 1.25, t["A"], bc.lda, stride, t["B"], bc.ldb,
                                          stride, 0.75, t["C"], bc.ldc, stride, bc.batch)
            else:
                call = lambda: generic_fn(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, t["alphas"], t["A"], t["a_off"], bc.lda,
                                          t["B"], t["b_off"], bc.ldb, t["betas"], t["C"], t["c_off"], bc.ldc, bc.batch)
            dev_graph, dev_eager = M.graph_timed(call, t["C"], steps, warmup)
            dev = min(dev_graph, dev_eager)
            nbytes = bc.algorithmic_bytes - (bc.batch * 32 if strided else 0)
            resident = sum(t[x].numel() * t[x].element_size() for x in ("A", "B", "C"))
            entry = {"workload": label, "gflops": round(bc.flops / dev / 1e9, 1), "ms": round(dev * 1e3, 5),
                     "ms_graph_replays": round(dev_graph * 1e3, 5), "ms_eager_launches": round(dev_eager * 1e3, 5),
                     "roofline": roofline("hbm", nbytes, dev, PEAK_HBM_GBS, label),
                     "note": "the faster of eager launches and replays of a HIP graph of 20 launches; "
                             + (f"{resident / 1e6:.0f} MB working set: repeated calls are served by the 256 MB last-level cache"
                                if resident < M.LAST_LEVEL_CACHE_BYTES else
                                (f"{resident / 1e6:.0f} MB working set: little more than the 256 MB last-level cache, which may still serve part of a repeated call"
                                 if resident < 1.5 * M.LAST_LEVEL_CACHE_BYTES else
                                 f"{resident / 1e6:.0f} MB working set: beyond the last-level cache, HBM-real"))}
            extra.append(entry)

        only_headline = args.only == "batched"
        for size in ((16,) if only_headline else (8, 16, 32, 64)):
            for batch in ((10000,) if only_headline else (1000, 10000)):
                batched_entry(f"sgemm_batched_f32_{batch}x{size}x{size}x{size}_gap7", W.config4_fast(size, batch))
        batched_entry("sgemm_strided_batched_f32_10000x16x16x16_gap7", W.config4_fast(16, 10000), strided=True)
        batched_entry("hgemm_batched_f16_10000x16x16x16_gap7", W.config4_fast(16, 10000, dtype="f16"))
        if not only_headline:
            batched_entry("hgemm_batched_f16_10000x64x64x64_gap7 (next row: FP16 storage; 328 MB moved)",
                          W.config4_fast(64, 10000, dtype="f16"))
            batched_entry("hgemm_batched_f16_20000x64x64x64_gap7 (the row above with twice the instances: 656 MB moved, HBM-real)",
                          W.config4_fast(64, 20000, dtype="f16"))
        # the HBM-real variant of the headline batched workload: sixteen times the instances (505 MB working set)
        batched_entry("sgemm_batched_f32_160000x16x16x16_gap7 (cold variant of 10000 x 16^3)", W.config4_fast(16, 160000))

    # ---- configuration 5: irregular and skinny FP32 shapes, op(A) = A^T, padded leading dimensions, beta = 1 -----
    if want("config5"):
        bounds = ("mfma", "mfma", "mfma", "hbm", "hbm", "hbm")
        for index, (m, n, k) in enumerate(W.CONFIG5_SHAPES):
            case = W.config5(index)
            small = m == 1 or n == 1 or m * n * k < 3e9
            gemm_entry(f"sgemm_f32_{m}x{n}x{k}_colmajor_TN_ldpad_beta1", case, bounds[index], small=small, cold=(m == 1 or n == 1))

    # ---- next row: convolution as IM2COL + GEMM on the layers whose GEMMs are the FP16 shapes of the metric's
    # workload list; microsecond-scale, so graph-timed like the batched calls
    if want("conv"):
        for index in range(len(W.CONV_LAYERS)):
            cc = W.conv_layer(index, "f16")
            geo = (cc.channels, cc.height, cc.width, cc.kernel, cc.pad, cc.stride, cc.dilation)
            im, wt, out = M.to_gpu(cc.im), M.to_gpu(cc.weights), M.to_gpu(cc.out)
            oh, ow = cc.out_hw
            col = torch.empty(cc.k * oh * ow, dtype=torch.float16, device="cuda")
            ws = torch.empty(max(G.mg_conv2d_workspace_bytes(G.MG_F16, *geo, cc.filters), 256), dtype=torch.uint8, device="cuda")
            t_unfold, _ = M.graph_timed(lambda: G.mg_him2col(*geo, im, col), col, steps, warmup)
            t_conv, t_conv_eager = M.graph_timed(lambda: G.mg_hconv2d(*geo, cc.filters, 1.0, im, wt, 0.0, out, ws), out,
                                                 steps, warmup)
            unfold_bytes = 2 * (cc.k * oh * ow + cc.channels * cc.height * cc.width)
            flops = 2.0 * cc.filters * oh * ow * cc.k
            extra.append({"workload": f"hconv2d_f16_c{cc.channels}_{cc.height}x{cc.width}_k{cc.kernel[0]}_s{cc.stride[0]}_f{cc.filters}"
                                      f" (GEMM {cc.filters}x{oh * ow}x{cc.k})",
                          "gflops": round(flops / t_conv / 1e9, 1), "ms": round(t_conv * 1e3, 5),
                          "ms_eager_launches": round(t_conv_eager * 1e3, 5), "ms_im2col": round(t_unfold * 1e3, 5),
                          "roofline_im2col": roofline("hbm", unfold_bytes, t_unfold, PEAK_HBM_GBS, None),
                          "note": "graph-timed; working set of a few MB, served by the last-level cache"})

    # ---- next row: the stand-alone matrix-vector product, a 1 GiB FP32 matrix (four times the last-level
    # cache) read once per call, in both operand orders
    if want("gemv"):
        size = 16384
        gen = torch.Generator(device="cuda").manual_seed(W.SEED_BASE)
        mat = torch.rand(size * size, dtype=torch.float32, device="cuda", generator=gen) - 0.5
        x = torch.rand(size, dtype=torch.float32, device="cuda", generator=gen) - 0.5
        y = torch.zeros(size, dtype=torch.float32, device="cuda")
        for trans, tag in ((W.NO_TRANS, "N"), (W.TRANS, "T")):
            need = G.mg_gemv_workspace_bytes(G.MG_F32, W.COL_MAJOR, trans, size, size, size)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None
            dev, _ = M.timed(lambda: G.mg_sgemv(W.COL_MAJOR, trans, size, size, 1.0, mat, size, x, 1, 0.0, y, 1, ws),
                             max(5, steps // 4), max(1, warmup // 4))
            label = f"sgemv_f32_{size}x{size}_colmajor_{tag}"
            extra.append({"workload": label, "gflops": round(2.0 * size * size / dev / 1e9, 1), "ms": round(dev * 1e3, 5),
                          "roofline": roofline("hbm", 4.0 * size * size, dev, PEAK_HBM_GBS, label)})
        del mat

    # ---- next row: the GEMM-derived level-3 routines at the size of the headline product (FP16 storage);
    # flops are the useful ones of each routine (SYRK and TRMM compute a full product: twice that)
    if want("level3"):
        size = 4096
        l3 = {"symm": W.level3_case("symm", "f16", W.COL_MAJOR, size, size, side=W.LEFT, uplo=W.LOWER, case=1),
              "syrk": W.level3_case("syrk", "f16", W.COL_MAJOR, size, size, k=size, uplo=W.LOWER, case=2),
              "trmm": W.level3_case("trmm", "f16", W.COL_MAJOR, size, size, side=W.LEFT, uplo=W.LOWER, case=3)}
        useful = {"symm": 2.0 * size ** 3, "syrk": 1.0 * size ** 3, "trmm": 1.0 * size ** 3}
        for routine, lc in l3.items():
            A = M.to_gpu(lc.A)
            if routine == "symm":
                need = G.mg_symm_workspace_bytes(G.MG_F16, lc.layout, lc.side, size, size)
            elif routine == "syrk":
                need = G.mg_syrk_workspace_bytes(G.MG_F16, lc.layout, lc.trans, size, size)
            else:
                need = G.mg_trmm_workspace_bytes(G.MG_F16, lc.layout, lc.side, lc.trans, size, size)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
            if routine == "symm":
                B, Cd = M.to_gpu(lc.B), M.to_gpu(lc.C)
                call = lambda: G.mg_hsymm(lc.layout, lc.side, lc.uplo, size, size, 1.0, A, lc.lda, B, lc.ldb, 0.0, Cd, lc.ldc, ws)
            elif routine == "syrk":
                Cd = M.to_gpu(lc.C)
                call = lambda: G.mg_hsyrk(lc.layout, lc.uplo, lc.trans, size, size, 1.0, A, lc.lda, 0.0, Cd, lc.ldc, ws)
            else:
                # in place: every timed call gets the workload's B back first (untimed copy), since a few calls on their
                # own result overflow FP16 and the time does depend on the values (the part is power-bound)
                B0 = M.to_gpu(lc.B)
                B = B0.clone()
                call = lambda: G.mg_htrmm(lc.layout, lc.side, lc.uplo, lc.trans, lc.diag, size, size, 1.0, A, lc.lda, B, lc.ldb, ws)
            if routine == "trmm":
                dev = M.timed_each(call, lambda: B.copy_(B0), max(5, steps // 4), max(3, warmup // 2))
            else:
                M.ramp(call, 0.03)
                dev, _ = M.timed(call, max(5, steps // 4), max(1, warmup // 4))
            label = f"h{routine}_f16_{size}_colmajor_lower" + ("_left" if routine != "syrk" else f"_k{size}")
            entry = {"workload": label, "gflops": round(useful[routine] / dev / 1e9, 1), "ms": round(dev * 1e3, 5),
                     "roofline": roofline("mfma", useful[routine], dev, PEAK_TFLOPS["f16"], label),
                     "note": "useful flops of the routine; includes the support kernels"}
            extra.append(entry)

    if head is None:
        print(json.dumps({"workloads": extra, "probes": probes}))
        return
    case, dev = head["case"], head["dev"]
    line = {
        "metric": "GFLOPS (2MNK/t) & % MI355X peak: SGEMM/HGEMM 4096^3, batched 16^3 GEMM",
        "value": round(case.flops / dev / 1e9, 1),
        "unit": "GFLOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(dev * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "hgemm_f16_4096x4096x4096_colmajor_NN_alpha1_beta0", "kernel": head["sel"]["name"],
                   "storage": "f16", "accumulate": "f32", "host_ms_per_step": round(head["wall"] * 1e3, 5),
                   "ms_fastest_single_call": round(head["fastest"] * 1e3, 5)},
        "roofline": roofline("mfma", case.flops, dev, PEAK_TFLOPS["f16"], "hgemm_f16_4096x4096x4096_colmajor_NN_alpha1_beta0"),
        "cpu_baseline": head["cpu"],
        "probes": probes,
        "traffic_measured_at_commit": traffic.get("measured_at_commit"),
        "paper_context": PAPER_CONTEXT,
        "workloads": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
