"""Per-workgroup phase trace of one launch of the double-precision kernels (a diagnostic; needs an MI355X).

    python -m paper_2003_00532_amd.phase_trace --workload c4_rankk [--variant -1] [--epilogue-mode 0]

Builds (if needed) a second copy of the library with -DGEMM_PHASE_TRACE, in which wave 0 of every workgroup stores the
constant 100 MHz clock at entry, after its first stage barrier, after its K loop and at exit, the shader clock at entry
and exit, and the hardware id of the compute unit it ran on.  Prints how long the phases take, how many workgroups a
compute unit holds on average and how many of them are inside their K loop, the gap between a workgroup's exit and the
next one's entry on the same compute unit, and the shader clock the chip held.  Each stored mark costs the workgroup
about 1 to 2.5 us under load (a scalar load, a clock read and a store behind the matrix instructions of older waves), so
the phases before the K loop read longer than they are in the library proper; the untraced time is printed beside.
"""
import argparse
import ctypes
import os
import subprocess
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
TRACE_LIB = os.path.join(HERE, "libgemm_f64_trace.so")


def build_trace_library(force=False):
    from . import build as b
    src = os.path.join(b.CSRC, "gemm_f64.hip")
    if not force and os.path.exists(TRACE_LIB) and all(os.path.getmtime(TRACE_LIB) >= os.path.getmtime(p) for p in b.DEPENDS):
        return TRACE_LIB
    flags = [f for f in b.FLAGS] + ["-DGEMM_PHASE_TRACE", '-DGEMM_BUILD_ID="%s"' % b.source_digest()]
    res = subprocess.run([b.HIPCC, *flags, src, "-o", TRACE_LIB + ".tmp"], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in res.stderr.splitlines() if "recognized feature" not in l))
    os.replace(TRACE_LIB + ".tmp", TRACE_LIB)
    return TRACE_LIB


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c4_rankk")
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--epilogue-mode", type=int, default=0, help="0 automatic, 1 load-add-store, 2 additions in memory")
    ap.add_argument("--build-only", action="store_true")
    args = ap.parse_args()
    path = build_trace_library()
    if args.build_only:
        print(path)
        return
    import numpy as np
    import torch
    from . import synth
    lib = ctypes.CDLL(path)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.gemm_f64_ex.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ci]
    lib.gemm_debug_set_trace.argtypes = [vp]
    lib.gemm_f64_set_epilogue_mode.argtypes = [ci]
    lib.gemm_f64_choose_variant.argtypes = [i64, i64, i64, ci]
    lib.gemm_f64_variant_name.restype = ctypes.c_char_p
    w = synth.WORKLOADS[args.workload]
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    variant = args.variant if args.variant >= 0 else lib.gemm_f64_choose_variant(w.M, w.N, w.K, cus)
    vname = lib.gemm_f64_variant_name(variant).decode()
    bm, bn = (int(x) for x in vname.split("_")[1].split("x")[:2])
    blocks = -(-w.M // bm) * -(-w.N // bn)
    dA, dB, dC = synth.device_workload_inputs(w, seed=0)
    buf = torch.zeros(blocks * 8, dtype=torch.int64, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    lib.gemm_f64_set_epilogue_mode(args.epilogue_mode)

    def call():
        rc = lib.gemm_f64_ex(w.M, w.N, w.K, dA.data_ptr(), w.lda, dB.data_ptr(), w.ldb, dC.data_ptr(), w.ldc, st, variant)
        assert rc == 0, rc

    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.5:       # clock ramp
        for _ in range(10):
            call()
        torch.cuda.synchronize()
    n = 20 if w.flops > 1e11 else 50
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        call()
    e1.record()
    torch.cuda.synchronize()
    untraced = e0.elapsed_time(e1) / n
    lib.gemm_debug_set_trace(buf.data_ptr())
    call()
    torch.cuda.synchronize()
    lib.gemm_debug_set_trace(None)
    t = buf.cpu().numpy().reshape(blocks, 8).astype(np.int64)
    us = lambda col: (t[:, col] - t[:, 0].min()) * 0.01      # 100 MHz ticks -> microseconds since the first entry
    entry, first_barrier, k_end, exit_ = us(0), us(3), us(4), us(5)
    span = exit_.max()
    print("%s, variant %s, epilogue mode %d: %d workgroups; untraced %.4f ms per call (%.1f %% of 78.6 TFLOP/s); traced launch spans %.4f ms"
          % (w.name, vname, args.epilogue_mode, blocks, untraced, 100 * w.flops / (untraced * 1e-3) / 78.6e12, span * 1e-3))

    def row(name, d):
        print("  %-34s mean %8.2f  p10 %8.2f  p50 %8.2f  p90 %8.2f us" % (name, d.mean(), np.percentile(d, 10), np.percentile(d, 50), np.percentile(d, 90)))

    row("entry -> first stage barrier", first_barrier - entry)
    late = entry > 5.0
    if late.any() and (~late).any():
        # a workgroup that starts on a busy compute unit is the youngest wave on its SIMDs, and the SIMD serves older ones first
        print("    of which the %d workgroups that start in the first 5 us: mean %.2f us; the %d that start later, beside workgroups "
              "already in their K loops: mean %.2f us" % ((~late).sum(), (first_barrier - entry)[~late].mean(), late.sum(),
                                                            (first_barrier - entry)[late].mean()))
    row("K loop", k_end - first_barrier)
    row("epilogue (C update)", exit_ - k_end)
    row("whole life", exit_ - entry)
    hw = t[:, 7]
    hwid, xcc = hw & 0xffffffff, (hw >> 32) & 0xf
    cu_key = ((xcc * 8 + ((hwid >> 13) & 7)) * 2 + ((hwid >> 12) & 1)) * 16 + ((hwid >> 8) & 0xf)
    keys = np.unique(cu_key)
    gaps = []
    for k in keys:
        sel = cu_key == k
        ent, ext = np.sort(entry[sel]), np.sort(exit_[sel])
        first_round = int((ent < ent[0] + 5.0).sum())
        if len(ent) > first_round:
            gaps.append(ent[first_round:] - ext[:len(ent) - first_round])
    if gaps:
        row("exit -> next entry, same compute unit", np.concatenate(gaps))
    print("  compute units seen %d; workgroups resident per compute unit on average %.2f, of which inside their K loop %.2f"
          % (len(keys), (exit_ - entry).sum() / (span * len(keys)), (k_end - first_barrier).sum() / (span * len(keys))))
    # the ragged end: from the moment the chip holds fewer than 97 % of its usual number of workgroups
    grid = np.linspace(0.0, span, 400)
    resident = np.array([((entry <= g) & (exit_ > g)).sum() for g in grid])
    steady = float(np.median(resident[50:300]))
    if steady > 0:
        full = np.where(resident >= 0.97 * steady)[0]
        drain_from = grid[full.max()] if len(full) else 0.0
        unused = (steady - resident[grid >= drain_from]).clip(min=0).sum() * (grid[1] - grid[0]) / (steady * span)
        last_exit = np.array([exit_[cu_key == k].max() for k in keys])
        print("  the end: %d workgroups resident in the steady state; the chip empties over the last %.1f us (%.1f %% of the launch), "
              "%.1f %% of the launch's slot-time is unused there; a compute unit's last exit is %.1f us before the end on average"
              % (steady, span - drain_from, 100 * (span - drain_from) / span, 100 * unused, (span - last_exit).mean()))
    mhz = (t[:, 2] - t[:, 1]) / ((t[:, 5] - t[:, 0]) * 0.01)
    # the eight XCDs one by one: workgroup b runs on XCD b % 8, so each has the same number of tiles whatever its speed
    def own_peak(x):
        # what the XCD's share of the flops took, against the FP64 matrix rate of its compute units at the clock it held
        sel = xcc == x
        cus_x = len(np.unique(cu_key[sel]))
        return 100.0 * (w.flops * sel.sum() / blocks) / (exit_[sel].max() * 1e-6) / (cus_x * 4 * 32 * mhz[sel].mean() * 1e6)

    print("  per XCD (workgroups | mean K loop us | last exit us | shader clock MHz | % of its own peak at that clock): " +
          "  ".join("%d: %d | %.1f | %.1f | %.0f | %.1f" % (x, (xcc == x).sum(), (k_end - first_barrier)[xcc == x].mean(),
                                                           exit_[xcc == x].max(), mhz[xcc == x].mean(), own_peak(x)) for x in np.unique(xcc)))
    print("  shader clock over workgroup lifetimes: mean %.0f MHz (p10 %.0f, p90 %.0f)" % (mhz.mean(), np.percentile(mhz, 10), np.percentile(mhz, 90)))


if __name__ == "__main__":
    main()
