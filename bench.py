#!/usr/bin/env python3
"""Benchmark of the fp64 GEMM hot path on one MI355X.

A step is one call of gemm_f64 (C += A B through the C ABI) on the named workload with A, B and C
already resident in HBM.  Prints ONE JSON line on stdout: DGEMM GFLOP/s = 2 M N K / t / 1e9 (the
paper's convention, Section 1.3), the roofline of the kernel (FP64 MFMA, 78.6 TFLOP/s published
peak; per-launch duration measured with HIP events on the launch stream) and the CPU oracle timed on
a bounded sample of the same workload.  Diagnostics go to stderr.  With --dtype f32 the same is
done for the single-precision path (gemm_f32, FP32 MFMA peak 157.3 TFLOP/s, float32 oracle).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_8192] [--variant -1] [--dtype f64|f32]
    python bench.py --copy-calibration     # plain device copy of known size, for scaling rocprof counters
    python bench.py --compare-vendor       # adds the vendor BLAS (torch.addmm) timed on the same buffers, as context
    python bench.py --workload c1_2048 --cold-cache   # adds the same call rotated over > 1 GiB of distinct operand sets
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP64_MFMA_TFLOPS = 78.6   # MI355X published dense FP64 matrix peak (256 CU x 128 flop/clk x 2.4 GHz)
PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X published dense FP32 matrix peak
PEAK_HBM_GBS = 8000.0

# The paper's own framing (context, not the target): its machine, the peak it prices against and its best result.
PAPER_CONTEXT = {
    "machine": "one core of an Intel Core i7-8700K (AVX-2, two FMA units, 4.7 GHz turbo), fp64",
    "peak_gflops_per_core": 75.2,            # Section 1.2
    "best_gflops": 61.94,                    # Section 2.10: 82 % of that peak, within 9 % of MKL / OpenBLAS
    "naive_gflops": [0.47, 4.53],            # Section 1.3: clang -O3 and gcc -O3 on the plain nest
    "workload": "C += A*B, M = 2088, N = K = 2048, row-major, single thread",
    "note": "another machine and another kind of hardware: context only, never a baseline for vs_baseline",
}


def traffic_from_profile(prec_letter, vname, wname, current_build_id):
    """HBM bytes per launch from the tracked rocprofv3 --pmc summary of this kernel and workload, if there is one.

    The summary (profiles/<s|d>gemm_<variant>_<workload>_pmc.txt) records FETCH_SIZE and WRITE_SIZE per dispatch,
    the copy-kernel scaling, the resulting bytes (a line `traffic_bytes_per_launch = N`) and the build id of the
    library it was taken with (`library_build_id = X`).  Returns (bytes or None, description of the source)."""
    import re
    path = os.path.join(ROOT, "profiles", "%sgemm_%s_%s_pmc.txt" % (prec_letter, vname, wname))
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text, re.M)
    b = re.search(r"^library_build_id\s*=\s*(\S+)", text, re.M)
    if not m:
        return None, None
    prof_id = b.group(1) if b else None
    return float(m.group(1)), {"file": os.path.relpath(path, ROOT), "profile_build_id": prof_id,
                               "current_build_id": current_build_id, "same_build": prof_id == current_build_id,
                               "what": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per dispatch, scaled by a plain copy; "
                                       "taken in a separate run, not in this one"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(w, seed, target_seconds=12.0, np_dtype=None):
    """Time the CPU oracle, as it stands, on complete rows of the same workload (all host threads)."""
    import numpy as np
    import oracle
    from paper_2003_00532_amd import synth

    np_dtype = np.float64 if np_dtype is None else np_dtype
    ref = oracle.gemm_f32_ref if np_dtype == np.float32 else oracle.gemm_f64_ref
    threads = oracle.ref_threads()
    _, B = synth.matrix(seed, synth.TAG_B, w.K, w.N, w.ldb, "uniform", np_dtype)

    def run(rows):
        A = np.empty((rows, w.K), np_dtype); synth.fill(A, seed, synth.TAG_A, "uniform")
        C = np.empty((rows, w.N), np_dtype); synth.fill(C, seed, synth.TAG_C, "uniform" if w.c_kind == "uniform" else "zeros")
        t0 = time.perf_counter()
        ref(A, B, C)
        return time.perf_counter() - t0

    pilot_rows = min(w.M, 4 * threads)
    t_pilot = run(pilot_rows)
    rows = int(pilot_rows * target_seconds / max(t_pilot, 1e-6))
    rows = max(pilot_rows, min(w.M, (rows // threads) * threads))
    t = run(rows)
    gflops = 2.0 * rows * w.N * w.K / t / 1e9
    # the paper's own numbers are single-core (Section 1.3): the same oracle on one thread, for about three seconds
    rows1 = max(1, min(w.M, int(3.0 * rows / t / threads)))
    oracle.set_ref_threads(1)
    try:
        t1 = run(rows1)
    finally:
        oracle.set_ref_threads(threads)
    return {"value": round(gflops, 3), "unit": "GFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "first %d of %d rows of %s (N=%d, K=%d) in %.2f s; full-size time extrapolates to %.0f s"
                      % (rows, w.M, w.name, w.N, w.K, t, t * w.M / rows),
            "single_thread": {"value": round(2.0 * rows1 * w.N * w.K / t1 / 1e9, 3), "unit": "GFLOP/s", "cores": 1,
                              "sample": "first %d rows in %.2f s" % (rows1, t1)}}


def copy_calibration():
    """A plain device-to-device copy of known size; run under rocprofv3 --pmc to scale FETCH_SIZE / WRITE_SIZE."""
    import torch
    n = 1 << 28  # 256 MiB read, 256 MiB written per copy
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "copies": 5}))


def time_launches(call, stream, launches):
    """Per-launch durations from HIP events recorded on the launch stream between consecutive launches (ms), and the
    duration per launch of the same number of launches back to back with one event on either side."""
    import torch
    events = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
    torch.cuda.synchronize()
    events[0].record(stream)
    for i in range(launches):
        call()
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    sep = [events[i].elapsed_time(events[i + 1]) for i in range(launches)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(launches):
        call()
    e1.record(stream)
    torch.cuda.synchronize()
    return sep, e0.elapsed_time(e1) / launches


OTHER_WORKLOADS = (("c0_256", 200), ("c1_2048", 50), ("c2_edge", 50), ("c4_rankk", 20))


def other_workloads(gemm_ex, choose, variant_name, np_dtype, peak, seed, stream, cus, skip):
    """The configurations that are not the headline: a handful of launches each of the automatic variant, inputs
    generated on the device by the same counter-based generator (same bits as the host one), timed both ways."""
    import torch
    from paper_2003_00532_amd import synth
    out = {}
    for name, launches in OTHER_WORKLOADS:
        if name == skip:
            continue
        w = synth.WORKLOADS[name]
        dA, dB, dC = synth.device_workload_inputs(w, seed=seed, dtype=np_dtype)

        def call():
            gemm_ex(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc, stream=stream, variant=-1)

        # warm-up by time, not by count: after an idle stretch the chip takes tens of milliseconds of load to reach
        # its clock (the first launches of a 0.25 ms kernel run up to 25 % slower)
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.5:
            for _ in range(10):
                call()
            torch.cuda.synchronize()
        sep, b2b = time_launches(call, stream, launches)
        ms = sum(sep) / len(sep)
        out[name] = {"kernel_variant": variant_name(choose(w.M, w.N, w.K, cus)), "launches": launches,
                     "kernel_ms": round(ms, 5), "kernel_ms_min": round(min(sep), 5),
                     "tflops": round(w.flops / (ms * 1e-3) / 1e12, 3), "frac": round(w.flops / (ms * 1e-3) / 1e12 / peak, 4),
                     "back_to_back_ms": round(b2b, 5), "back_to_back_tflops": round(w.flops / (b2b * 1e-3) / 1e12, 3),
                     "back_to_back_frac": round(w.flops / (b2b * 1e-3) / 1e12 / peak, 4)}
        from paper_2003_00532_amd import binding as _b
        import numpy as np
        f32w = np_dtype == np.float32
        # HBM-side bytes per launch from the tracked counter summary of this kernel and workload, if there is one
        traffic, source = traffic_from_profile("s" if f32w else "d", out[name]["kernel_variant"], name, _b.gemm_f64_build_id())
        if traffic is not None:
            out[name]["traffic"] = traffic
            out[name]["algorithmic_bytes_per_launch"] = w.algorithmic_bytes * np.dtype(np_dtype).itemsize / 8.0
            out[name]["traffic_source"] = {"file": source.get("file"), "same_build": source.get("same_build")}
        # the same workload through the entry point that takes a workspace, when its plan would use one
        ws_bytes = (_b.gemm_f32_split_k_workspace_bytes if f32w else _b.gemm_f64_split_k_workspace_bytes)(0, 0, w.M, w.N, w.K, cus)
        if ws_bytes > 0:
            general_ws = _b.gemm_f32_general_ws if f32w else _b.gemm_f64_general_ws
            workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dA.device)

            def call_ws():
                general_ws(0, 0, w.M, w.N, w.K, 1.0, dA, w.lda, dB, w.ldb, 1.0, dC, w.ldc, workspace, ws_bytes, stream=stream)

            for _ in range(10):
                call_ws()
            sep_ws, b2b_ws = time_launches(call_ws, stream, launches)
            tplan = (_b.gemm_f32_tail_split_plan if f32w else _b.gemm_f64_tail_split_plan)(0, 0, w.M, w.N, w.K, cus)
            out[name]["with_workspace"] = {
                "entry_point": "general_ws, alpha = beta = 1", "workspace_bytes": ws_bytes, "kernel_variant": variant_name(tplan[0]),
                "tail_split": {"tiles": tplan[1], "slices": tplan[2], "k_chunk": tplan[3]},
                "ms": round(sum(sep_ws) / len(sep_ws), 5), "frac": round(w.flops / (sum(sep_ws) / len(sep_ws) * 1e-3) / 1e12 / peak, 4),
                "back_to_back_ms": round(b2b_ws, 5), "back_to_back_frac": round(w.flops / (b2b_ws * 1e-3) / 1e12 / peak, 4)}
            del workspace
        log("%s: %s" % (name, json.dumps(out[name])))
        del dA, dB, dC
    return out


STUDY_SHAPES = [(256, 256, 256), (512, 512, 512), (1024, 1024, 1024), (1536, 1536, 1536), (2048, 2048, 2048), (3000, 3000, 3000),
                (4096, 4096, 4096), (2088, 2049, 2047), (8192, 8192, 8192), (16384, 16384, 256), (1024, 8192, 512),
                (8192, 1024, 4096), (300, 300, 300), (5000, 200, 3000), (640, 640, 8192), (6144, 6144, 1024), (2304, 2304, 2304)]


def selection_study(f32, stream, cus):
    """How good is the shape-driven variant choice?  Every tiled variant timed on 17 shapes (dense, seeded uniform
    operands, calls back to back after a warm-up by time); the regret of a shape is the time of the variant the
    selection rule picks over the time of the best variant, minus one."""
    import torch
    from paper_2003_00532_amd import binding
    gemm_ex = binding.gemm_f32_ex if f32 else binding.gemm_f64_ex
    choose = binding.gemm_f32_choose_variant if f32 else binding.gemm_f64_choose_variant
    name = binding.gemm_f32_variant_name if f32 else binding.gemm_f64_variant_name
    peak = PEAK_FP32_MFMA_TFLOPS if f32 else PEAK_FP64_MFMA_TFLOPS
    tdt = torch.float32 if f32 else torch.float64
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(0)
    rows, total = [], 0.0
    for (M, N, K) in STUDY_SHAPES:
        dA = torch.rand((M, K), dtype=tdt, device="cuda:0", generator=gen) * 2 - 1
        dB = torch.rand((K, N), dtype=tdt, device="cuda:0", generator=gen) * 2 - 1
        dC = torch.zeros((M, N), dtype=tdt, device="cuda:0")
        flops = 2.0 * M * N * K
        reps = max(5, min(300, int(1.5e12 / flops)))
        times = {}
        for v in (1, 2, 3, 4, 5):
            def call():
                gemm_ex(M, N, K, dA, K, dB, N, dC, N, stream=stream, variant=v)
            t0 = time.perf_counter()
            while time.perf_counter() - t0 < 0.2:
                for _ in range(5):
                    call()
                torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                call()
            e1.record(stream)
            torch.cuda.synchronize()
            times[v] = e0.elapsed_time(e1) / reps
        chosen = choose(M, N, K, cus)
        best = min(times, key=times.get)
        regret = times[chosen] / times[best] - 1.0
        total += regret
        rows.append({"shape": [M, N, K], "chosen": name(chosen), "chosen_ms": round(times[chosen], 5),
                     "chosen_frac": round(flops / (times[chosen] * 1e-3) / 1e12 / peak, 4), "best": name(best),
                     "best_ms": round(times[best], 5), "regret": round(regret, 4),
                     "all_ms": {name(v): round(t, 5) for v, t in times.items()}})
        log("%-18s chosen %-16s %9.4f ms (%5.1f %%) | best %-16s %9.4f ms | regret %4.1f %% | %s" % (
            "%dx%dx%d" % (M, N, K), name(chosen), times[chosen], 100 * rows[-1]["chosen_frac"], name(best), times[best], 100 * regret,
            " ".join("%s:%.4f" % (name(v).replace("mfma_", ""), t) for v, t in times.items())))
    log("mean regret %.2f %%, largest %.2f %%" % (100 * total / len(rows), 100 * max(r["regret"] for r in rows)))
    return {"dtype": "f32" if f32 else "f64", "mean_regret": round(total / len(rows), 4), "max_regret": max(r["regret"] for r in rows), "shapes": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3_8192")
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--dtype", choices=["f64", "f32"], default="f64")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short timings of the configurations that are not the headline")
    ap.add_argument("--with-workspace", action="store_true",
                    help="time gemm_*_general_ws (alpha = beta = 1) with the workspace its plan asks for instead of gemm_*_ex: "
                         "the k range, or the k range of the last tiles only, may then be split")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--selection-study", action="store_true",
                    help="instead of the benchmark: time every tiled variant on 17 shapes and report the regret of the selection rule")
    ap.add_argument("--compare-vendor", action="store_true",
                    help="after the measurement, time the vendor BLAS behind torch.addmm on the same buffers (context only)")
    ap.add_argument("--cold-cache", action="store_true",
                    help="after the measurement, time the same call rotated over distinct operand sets of more than "
                         "1 GiB in total, so that no call finds its operands in the 256 MiB last-level cache")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by row blocks "
            "without collectives, see DESIGN.md, but no multi-GPU figure is produced)" % args.gpus)
        sys.exit(2)

    import torch
    from paper_2003_00532_amd import binding, synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(1)
    binding.load()
    if args.copy_calibration:
        copy_calibration()
        return
    if args.selection_study:
        print(json.dumps(selection_study(args.dtype == "f32", torch.cuda.current_stream(),
                                         torch.cuda.get_device_properties(0).multi_processor_count)), flush=True)
        return

    import numpy as np
    f32 = args.dtype == "f32"
    np_dtype = np.float32 if f32 else np.float64
    gemm_ex = binding.gemm_f32_ex if f32 else binding.gemm_f64_ex
    choose = binding.gemm_f32_choose_variant if f32 else binding.gemm_f64_choose_variant
    variant_name = binding.gemm_f32_variant_name if f32 else binding.gemm_f64_variant_name
    peak = PEAK_FP32_MFMA_TFLOPS if f32 else PEAK_FP64_MFMA_TFLOPS
    elem = 4 if f32 else 8

    w = synth.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    t0 = time.perf_counter()
    dA, dB, dC = synth.device_workload_inputs(w, seed=args.seed, dtype=np_dtype, device=dev)
    torch.cuda.synchronize()
    log("inputs for %s generated and resident in HBM after %.1f s" % (w.name, time.perf_counter() - t0))

    props = torch.cuda.get_device_properties(0)
    variant = args.variant if args.variant >= 0 else choose(w.M, w.N, w.K, props.multi_processor_count)
    vname = variant_name(variant)

    stream = torch.cuda.current_stream()

    ws_plan = None
    if args.with_workspace:
        general_ws = binding.gemm_f32_general_ws if f32 else binding.gemm_f64_general_ws
        cus = props.multi_processor_count
        ws_bytes = (binding.gemm_f32_split_k_workspace_bytes if f32 else binding.gemm_f64_split_k_workspace_bytes)(0, 0, w.M, w.N, w.K, cus)
        workspace = torch.empty(max(1, ws_bytes), dtype=torch.uint8, device=dev)
        sv, splits, chunk = (binding.gemm_f32_split_k_plan if f32 else binding.gemm_f64_split_k_plan)(0, 0, w.M, w.N, w.K, cus)
        tv, ttiles, tsplits, tchunk = (binding.gemm_f32_tail_split_plan if f32 else binding.gemm_f64_tail_split_plan)(0, 0, w.M, w.N, w.K, cus)
        variant = tv
        vname = variant_name(variant)
        ws_plan = {"workspace_bytes": ws_bytes, "split_k": {"slices": splits, "k_chunk": chunk},
                   "tail_split": {"tiles": ttiles, "slices": tsplits, "k_chunk": tchunk}}

    def step():
        if args.with_workspace:
            general_ws(0, 0, w.M, w.N, w.K, 1.0, dA, w.lda, dB, w.ldb, 1.0, dC, w.ldc, workspace, ws_bytes, stream=stream)
        else:
            gemm_ex(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc, stream=stream, variant=args.variant)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # short kernels: keep warming until the chip has been under load for half a second (clock ramp), see other_workloads
    t0 = time.perf_counter()
    while w.flops < 1e11 and time.perf_counter() - t0 < 0.5:
        for _ in range(10):
            step()
        torch.cuda.synchronize()

    # whole-job wall time over exactly `steps` steps, and per-launch durations from HIP events recorded
    # on the launch stream (event i sits between launch i-1 and launch i)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record(stream)
    for i in range(args.steps):
        step()
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_launch_ms = [events[i].elapsed_time(events[i + 1]) for i in range(args.steps)]
    kernel_ms = sum(per_launch_ms) / len(per_launch_ms)
    kernel_ms_median = sorted(per_launch_ms)[len(per_launch_ms) // 2]

    # the same number of launches back to back, one event on either side (how a caller would stream them): for short
    # kernels the event records between launches above cost a few per cent
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    back_to_back_ms = e0.elapsed_time(e1) / args.steps

    ms_per_step = wall * 1e3 / args.steps
    gflops = w.flops / (ms_per_step * 1e-3) / 1e9
    achieved_tflops = w.flops / (kernel_ms * 1e-3) / 1e12
    traffic, traffic_source = traffic_from_profile("s" if f32 else "d", vname, w.name, binding.gemm_f64_build_id())
    alg_bytes = w.algorithmic_bytes * elem / 8.0
    prec = "fp32" if f32 else "fp64"

    out = {
        "metric": "%sGEMM GFLOP/s (2MNK/t), 1 GPU" % ("S" if f32 else "D"),
        "value": round(gflops, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: %s row-major C += A*B, M=%d N=%d K=%d, lda=%d ldb=%d ldc=%d, A,B uniform[-1,1) seed %d, C %s"
                               % (w.name, prec, w.M, w.N, w.K, w.lda, w.ldb, w.ldc, args.seed, w.c_kind),
                   "kernel_variant": vname, "device": props.name, "compute_units": props.multi_processor_count,
                   "library_build_id": binding.gemm_f64_build_id()},
        "pct_of_%s_mfma_peak" % prec: round(100.0 * gflops / (peak * 1e3), 2),
        "roofline": {"bound": "mfma", "achieved": round(achieved_tflops, 3), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved_tflops / peak, 4),
                     "traffic": traffic, "traffic_source": traffic_source, "kernel_ms": round(kernel_ms, 4),
                     "kernel_ms_min": round(min(per_launch_ms), 4), "kernel_ms_median": round(kernel_ms_median, 4),
                     "kernel_ms_max": round(max(per_launch_ms), 4), "back_to_back_ms": round(back_to_back_ms, 4),
                     "back_to_back_frac": round(w.flops / (back_to_back_ms * 1e-3) / 1e12 / peak, 4),
                     "algorithmic_flops_per_launch": w.flops, "algorithmic_bytes_per_launch": alg_bytes},
    }
    if ws_plan is not None:
        out["config"]["entry_point"] = "gemm_%s_general_ws(0, 0, ..., alpha = 1, ..., beta = 1, ..., workspace)" % args.dtype
        out["config"]["workspace_plan"] = ws_plan
    # The peak recomputed from what the device reports (compute units x 4 SIMDs x flops per MFMA / issue cycles x clock)
    cus, clock_khz, peak64, peak32 = binding.gemm_f64_device_peak()
    out["roofline"]["peak_from_device_props"] = round(peak32 if f32 else peak64, 2)
    out["config"]["clock_mhz"] = clock_khz / 1e3
    # What the matrix pipes sustain with no memory traffic at the clock the chip holds (the library's MFMA-only
    # probe), reported beside the published peak: the kernel's distance from the hardware, not from the data sheet.
    probe = binding.gemm_f32_mfma_probe if f32 else binding.gemm_f64_mfma_probe
    sink = torch.empty(512 * props.multi_processor_count, dtype=torch.float32 if f32 else torch.float64, device=dev)
    iters = 40000 if f32 else 20000
    probe(iters, sink, sink.numel(), stream=stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    probe_flops = probe(iters, sink, sink.numel(), stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    mfma_only = probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    out["roofline"]["mfma_only_tflops"] = round(mfma_only, 2)
    out["roofline"]["frac_of_mfma_only"] = round(achieved_tflops / mfma_only, 4)
    if args.cold_cache:
        # Repeated calls on one operand set of a small workload are served from the last-level cache (256 MiB); here
        # consecutive calls use different sets, more than 1 GiB in all, so every call starts from HBM.
        set_bytes = (dA.numel() + dB.numel() + dC.numel()) * elem
        n_sets = max(2, -(-(1 << 30) // set_bytes) + 1)
        sets = [(dA.clone(), dB.clone(), dC.clone()) for _ in range(n_sets)]
        calls = n_sets * max(1, min(args.steps, 200) // n_sets)

        def cold_round():
            for i in range(calls):
                a, b, c = sets[i % n_sets]
                gemm_ex(w.M, w.N, w.K, a, w.lda, b, w.ldb, c, w.ldc, stream=stream, variant=args.variant)

        cold_round()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        cold_round()
        e1.record(stream)
        torch.cuda.synchronize()
        cms = e0.elapsed_time(e1) / calls
        out["cold_cache"] = {"value": round(w.flops / (cms * 1e-3) / 1e9, 1), "unit": "GFLOP/s", "ms_per_call": round(cms, 4),
                             "operand_sets": n_sets, "bytes_per_set": set_bytes, "calls": calls,
                             "frac": round(w.flops / (cms * 1e-3) / 1e12 / peak, 4)}
        del sets
    if args.compare_vendor:
        # Context, never the product path: the library routine behind torch.addmm (rocBLAS / hipBLASLt) on the
        # same operands, timed the same way after the measurement above is complete (dense views only).
        if w.lda == w.K and w.ldb == w.N and w.ldc == w.N:
            n = max(3, min(args.steps, 20))
            for _ in range(3):
                torch.addmm(dC, dA, dB, out=dC)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(n):
                torch.addmm(dC, dA, dB, out=dC)
            e1.record(stream)
            torch.cuda.synchronize()
            vms = e0.elapsed_time(e1) / n
            out["vendor_blas_context"] = {"value": round(w.flops / (vms * 1e-3) / 1e9, 1), "unit": "GFLOP/s",
                                          "ms_per_call": round(vms, 4), "what": "torch.addmm on the same buffers, comparison only"}
        else:
            out["vendor_blas_context"] = None
    out["paper_context"] = PAPER_CONTEXT
    if not args.no_other_workloads:
        del dA, dB, dC
        out["other_workloads"] = other_workloads(gemm_ex, choose, variant_name, np_dtype, peak, args.seed, stream,
                                                 props.multi_processor_count, w.name)
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        out["cpu_baseline"] = cpu_baseline(w, args.seed, np_dtype=np_dtype)
        log("cpu baseline took %.1f s" % (time.perf_counter() - t0))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
