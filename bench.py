"""Benchmark of the GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" is one mg_hgemm call on the headline workload: FP16 storage / FP32 accumulation,
column-major, op(A)=A, op(B)=B, m=n=k=4096, alpha=1, beta=0, entries N(0, K^-1/2) rounded to
FP16 (seeded, synthetic).  Inputs are resident in HBM before the timed region; W warm-up
steps, then exactly K steps between two device synchronisations.  Prints ONE JSON line:
GFLOPS = 2mnk/t, the MFMA roofline of the kernel, the CPU oracle timed on a bounded sample of
the same workload (cpu_baseline), and -- measured the same way right after -- the other two
workloads of the metric (SGEMM 4096^3 and batched 10000 x 16^3) under "workloads".
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

# HBM traffic per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain copy kernel of known size (profiles/ holds the summaries these come from).
MEASURED_TRAFFIC_BYTES = {"hgemm_4096": 235042978, "sgemm_4096": 470094977, "batched_16x10000": 42897824,
                          "sgemv_16384_N": 1075332914, "sgemv_16384_T": 1074414473}


def timed(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - wall0) / steps
    dev = start.elapsed_time(stop) * 1e-3 / steps          # HIP events on the stream the kernels run on
    return dev, wall


def graph_timed(call, c_buffer, steps, warmup, per_graph=20):
    """Device time per call of a microsecond-scale launch: shorter than the host can issue launches (about
    8 us per call from Python), so the call is captured once into a HIP graph of `per_graph` launches and the
    graph is replayed; the events then bracket back-to-back kernels.  Every replay of a one-launch graph is
    first checked against the eager result.  Returns (seconds per call from replays, from eager launches)."""
    import torch
    c0 = c_buffer.clone()
    call()
    eager = c_buffer.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()                                       # warm-up on a capture-capable stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(per_graph):
            call()
    one = torch.cuda.CUDAGraph()
    with torch.cuda.graph(one):
        call()
    for _ in range(3):
        c_buffer.copy_(c0)
        one.replay()
        torch.cuda.synchronize()
        assert torch.equal(c_buffer, eager), "graph replay differs from the eager call"
    dev, _ = timed(graph.replay, max(1, steps // 2), max(1, warmup // 4))
    dev_eager, _ = timed(call, steps, warmup)
    return dev / per_graph, dev_eager


def gemm_workload(G, case, steps, warmup):
    import torch
    from tests import helpers as H
    fn = G.mg_sgemm if case.dtype == "f32" else G.mg_hgemm
    code = G.MG_F32 if case.dtype == "f32" else G.MG_F16
    A, B, C = H.to_gpu(case.A), H.to_gpu(case.B), H.to_gpu(case.C)
    need = G.mg_gemm_workspace_bytes(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda,
                                     case.ldb, case.ldc)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None
    sel = G.mg_query_selected(code, case.layout, case.ta, case.tb, case.m, case.n, case.k, case.lda, case.ldb,
                              case.ldc, case.alpha, case.beta)

    def call():
        fn(case.layout, case.ta, case.tb, case.m, case.n, case.k, case.alpha, A, case.lda, B, case.ldb, case.beta,
           C, case.ldc, ws)

    dev, wall = timed(call, steps, warmup)
    return dev, wall, sel, C


def roofline_mfma(case, seconds, key):
    tf = case.flops / seconds / 1e12
    peak = PEAK_TFLOPS[case.dtype]
    return {"bound": "mfma", "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s",
            "frac": round(tf / peak, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(key)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--only", default=None, help="hgemm | sgemm | batched | conv | gemv | level3 | copy: run a single workload (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    from paper_1705_05249_amd import gemm as G, workloads as W
    from tests import helpers as H
    G.lib()
    G.mg_clear_override()
    steps, warmup = args.steps, args.warmup
    extra = []

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
    if args.only in (None, "hgemm"):
        case = W.config3(4)
        dev, wall, sel, C = gemm_workload(G, case, steps, warmup)
        head = {"case": case, "dev": dev, "wall": wall, "sel": sel}
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
            err = H.rel_error(got, c_ref, d_ref)
            assert err <= H.TOL["f16"], f"benchmark output fails parity: {err}"
            cpu = {"value": round(2.0 * case.k * rows.size / t_cpu / 1e9, 3), "unit": "GFLOPS",
                   "cores": gemm_oracle.threads(), "kind": "oracle",
                   "sample": f"{rows.size} of {case.m * case.n} output entries (256 full rows, 256 full columns, "
                             f"8192 scattered), each a full k={case.k} FP64 dot product; {t_cpu:.1f} s",
                   "max_rel_err_gpu_vs_oracle": float(f"{err:.3e}")}
        head["cpu"] = cpu

    # ---- the other two workloads of the metric ----------------------------------------------------
    if args.only in (None, "sgemm"):
        logical = W.config2_logical(4096)
        case = W.config2_variant(4096, W.COL_MAJOR, W.NO_TRANS, W.NO_TRANS, 0.0, logical)
        dev, wall, sel, _ = gemm_workload(G, case, max(5, steps // 5), max(1, warmup // 2))
        extra.append({"workload": "sgemm_f32_4096x4096x4096_colmajor_NN_beta0", "gflops": round(case.flops / dev / 1e9, 1),
                      "ms": round(dev * 1e3, 4), "kernel": sel["name"], "roofline": roofline_mfma(case, dev, "sgemm_4096")})
        del logical
    if args.only in (None, "batched"):
        bc = W.config4_fast(16, 10000)
        t = {name: H.to_gpu(getattr(bc, name)) for name in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}
        stride = int(bc.a_off[1] - bc.a_off[0])

        def generic():
            G.mg_sgemm_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, t["alphas"], t["A"], t["a_off"], bc.lda,
                               t["B"], t["b_off"], bc.ldb, t["betas"], t["C"], t["c_off"], bc.ldc, bc.batch)

        def strided():
            G.mg_sgemm_strided_batched(bc.layout, bc.ta, bc.tb, bc.m, bc.n, bc.k, 1.25, t["A"], bc.lda, stride, t["B"],
                                       bc.ldb, stride, 0.75, t["C"], bc.ldc, stride, bc.batch)

        note = ("timed as replays of a HIP graph of 20 launches (host launch rate is ~8 us/call); "
                "41 MB working set: repeated calls are served by the 256 MB last-level cache")
        for label, call, scalar_bytes in (("sgemm_batched_f32_10000x16x16x16_gap7", generic, 32),
                                          ("sgemm_strided_batched_f32_10000x16x16x16_gap7", strided, 0)):
            dev, dev_eager = graph_timed(call, t["C"], steps, warmup)
            nbytes = bc.algorithmic_bytes - bc.batch * (32 - scalar_bytes)
            gbs = nbytes / dev / 1e9
            extra.append({"workload": label, "gflops": round(bc.flops / dev / 1e9, 1), "ms": round(dev * 1e3, 5),
                          "ms_eager_launches": round(dev_eager * 1e3, 5),
                          "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": round(gbs / PEAK_HBM_GBS, 4),
                                       "traffic": MEASURED_TRAFFIC_BYTES.get("batched_16x10000") if scalar_bytes else None},
                          "note": note})

    # ---- next row: the batched workload in FP16 storage
    if args.only in (None, "batched"):
        hb = W.config4_fast(16, 10000, dtype="f16")
        th = {name: H.to_gpu(getattr(hb, name)) for name in ("A", "B", "C", "a_off", "b_off", "c_off", "alphas", "betas")}

        def half_generic():
            G.mg_hgemm_batched(hb.layout, hb.ta, hb.tb, hb.m, hb.n, hb.k, th["alphas"], th["A"], th["a_off"], hb.lda,
                               th["B"], th["b_off"], hb.ldb, th["betas"], th["C"], th["c_off"], hb.ldc, hb.batch)

        dev, dev_eager = graph_timed(half_generic, th["C"], steps, warmup)
        gbs = hb.algorithmic_bytes / dev / 1e9
        extra.append({"workload": "hgemm_batched_f16_10000x16x16x16_gap7", "gflops": round(hb.flops / dev / 1e9, 1),
                      "ms": round(dev * 1e3, 5), "ms_eager_launches": round(dev_eager * 1e3, 5),
                      "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                   "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None},
                      "note": "graph-timed; 21 MB working set, served by the last-level cache"})

    # ---- next row: convolution as IM2COL + GEMM on the layers whose GEMMs are the FP16 shapes of the metric's
    # workload list; microsecond-scale, so graph-timed like the batched calls
    if args.only in (None, "conv"):
        for index in range(len(W.CONV_LAYERS)):
            cc = W.conv_layer(index, "f16")
            geo = (cc.channels, cc.height, cc.width, cc.kernel, cc.pad, cc.stride, cc.dilation)
            im, wt, out = H.to_gpu(cc.im), H.to_gpu(cc.weights), H.to_gpu(cc.out)
            oh, ow = cc.out_hw
            col = torch.empty(cc.k * oh * ow, dtype=torch.float16, device="cuda")
            ws = torch.empty(max(G.mg_conv2d_workspace_bytes(G.MG_F16, *geo, cc.filters), 256), dtype=torch.uint8, device="cuda")
            t_unfold, _ = graph_timed(lambda: G.mg_him2col(*geo, im, col), col, steps, warmup)
            t_conv, t_conv_eager = graph_timed(lambda: G.mg_hconv2d(*geo, cc.filters, 1.0, im, wt, 0.0, out, ws), out,
                                               steps, warmup)
            unfold_bytes = 2 * (cc.k * oh * ow + cc.channels * cc.height * cc.width)
            gbs = unfold_bytes / t_unfold / 1e9
            flops = 2.0 * cc.filters * oh * ow * cc.k
            extra.append({"workload": f"hconv2d_f16_c{cc.channels}_{cc.height}x{cc.width}_k{cc.kernel[0]}_s{cc.stride[0]}_f{cc.filters}"
                                      f" (GEMM {cc.filters}x{oh * ow}x{cc.k})",
                          "gflops": round(flops / t_conv / 1e9, 1), "ms": round(t_conv * 1e3, 5),
                          "ms_eager_launches": round(t_conv_eager * 1e3, 5), "ms_im2col": round(t_unfold * 1e3, 5),
                          "roofline_im2col": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                              "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None},
                          "note": "graph-timed; working set of a few MB, served by the last-level cache"})

    # ---- next row: the stand-alone matrix-vector product, a 1 GiB FP32 matrix (four times the last-level
    # cache) read once per call, in both operand orders
    if args.only in (None, "gemv"):
        size = 16384
        gen = torch.Generator(device="cuda").manual_seed(W.SEED_BASE)
        mat = torch.rand(size * size, dtype=torch.float32, device="cuda", generator=gen) - 0.5
        x = torch.rand(size, dtype=torch.float32, device="cuda", generator=gen) - 0.5
        y = torch.zeros(size, dtype=torch.float32, device="cuda")
        for trans, tag in ((W.NO_TRANS, "N"), (W.TRANS, "T")):
            need = G.mg_gemv_workspace_bytes(G.MG_F32, W.COL_MAJOR, trans, size, size, size)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda") if need else None
            dev, _ = timed(lambda: G.mg_sgemv(W.COL_MAJOR, trans, size, size, 1.0, mat, size, x, 1, 0.0, y, 1, ws),
                           steps, warmup)
            gbs = 4.0 * size * size / dev / 1e9
            extra.append({"workload": f"sgemv_f32_{size}x{size}_colmajor_{tag}", "gflops": round(2.0 * size * size / dev / 1e9, 1),
                          "ms": round(dev * 1e3, 5),
                          "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": round(gbs / PEAK_HBM_GBS, 4),
                                       "traffic": MEASURED_TRAFFIC_BYTES.get(f"sgemv_{size}_{tag}")}})

    # ---- next row: the GEMM-derived level-3 routines at the size of the headline product (FP16 storage);
    # flops are the useful ones of each routine (SYRK and TRMM compute a full product: twice that)
    if args.only in (None, "level3"):
        size = 4096
        l3 = {"symm": W.level3_case("symm", "f16", W.COL_MAJOR, size, size, side=W.LEFT, uplo=W.LOWER, case=1),
              "syrk": W.level3_case("syrk", "f16", W.COL_MAJOR, size, size, k=size, uplo=W.LOWER, case=2),
              "trmm": W.level3_case("trmm", "f16", W.COL_MAJOR, size, size, side=W.LEFT, uplo=W.LOWER, case=3)}
        useful = {"symm": 2.0 * size ** 3, "syrk": 1.0 * size ** 3, "trmm": 1.0 * size ** 3}
        for routine, lc in l3.items():
            A = H.to_gpu(lc.A)
            ws = H.level3_workspace(lc)
            if routine == "symm":
                B, Cd = H.to_gpu(lc.B), H.to_gpu(lc.C)
                call = lambda: G.mg_hsymm(lc.layout, lc.side, lc.uplo, size, size, 1.0, A, lc.lda, B, lc.ldb, 0.0, Cd, lc.ldc, ws)
            elif routine == "syrk":
                Cd = H.to_gpu(lc.C)
                call = lambda: G.mg_hsyrk(lc.layout, lc.uplo, lc.trans, size, size, 1.0, A, lc.lda, 0.0, Cd, lc.ldc, ws)
            else:
                # in place: the operand shrinks or grows from call to call; the time does not depend on the values
                B = H.to_gpu(lc.B)
                call = lambda: G.mg_htrmm(lc.layout, lc.side, lc.uplo, lc.trans, lc.diag, size, size, 1.0, A, lc.lda, B, lc.ldb, ws)
            dev, _ = timed(call, steps, warmup)
            tf = useful[routine] / dev / 1e12
            extra.append({"workload": f"h{routine}_f16_{size}_colmajor_lower" + ("_left" if routine != "syrk" else f"_k{size}"),
                          "gflops": round(tf * 1e3, 1), "ms": round(dev * 1e3, 5),
                          "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_TFLOPS["f16"], "unit": "TFLOP/s",
                                       "frac": round(tf / PEAK_TFLOPS["f16"], 4), "traffic": None},
                          "note": "useful flops of the routine; includes the support kernels"})

    if head is None:
        print(json.dumps({"workloads": extra}))
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
        "dtype": "f16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "hgemm_f16_4096x4096x4096_colmajor_NN_alpha1_beta0", "kernel": head["sel"]["name"],
                   "host_ms_per_step": round(head["wall"] * 1e3, 5)},
        "roofline": roofline_mfma(case, dev, "hgemm_4096"),
        "cpu_baseline": head["cpu"],
        "workloads": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
