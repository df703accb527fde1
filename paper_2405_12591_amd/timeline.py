"""Time line of the matrix-core decode kernel's waves, from the instrumented build of the library.

    python -m paper_2405_12591_amd.timeline --build            # here (no GPU needed): builds libdecoquant_timeline.so
    python -m paper_2405_12591_amd.timeline --workload llama7b_4bit     # on the GPU
    python -m paper_2405_12591_amd.timeline --issue-probe               # on the GPU: do matrix and vector instructions overlap?

The instrumented build is the product's sources compiled with -DDQ_TIMELINE: every wave of
dq::decode_mfma_kernel stores the 100 MHz real-time counter at its entry, when its first tile's
arithmetic starts, at the start of each of its tiles, when its last tile is done and at its exit.  The
run below launches the decode call back to back (clocks settled, caches rotated as in bench.py), reads
out the time line of the last launch and prints, per event, the spread over the launch's waves, then
the median first-tile-to-last-tile time by XCD (workgroups go to the eight XCDs round-robin in launch
order).  The product library is not touched.

--issue-probe runs the instrumented build's other tool instead: loops of four independent matrix
instructions of one kind, sixteen independent fp32 FMAs, or both, four waves per SIMD, and prints
the time per loop body, which tells whether the two kinds of instruction run side by side.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true", help="build the instrumented library and stop")
    ap.add_argument("--issue-probe", action="store_true", help="time matrix and vector instruction streams, alone and together")
    ap.add_argument("--workload", default="llama7b_4bit")
    ap.add_argument("--launches", type=int, default=2000)
    ap.add_argument("--unit-map", type=int, default=None, help="DQ_DECODE_UNIT_MAP override (default: the library's choice)")
    args = ap.parse_args()
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    import importlib.util
    spec = importlib.util.spec_from_file_location("_dq_build", os.path.join(ROOT, "paper_2405_12591_amd", "build.py"))
    build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(build)
    if args.build or not os.path.exists(build.TIMELINE_LIB_PATH):
        print("built", build.build_library(timeline=True))
        if args.build:
            return
    import ctypes as C

    import numpy as np
    import torch

    import bench
    import paper_2405_12591_amd as dq
    from paper_2405_12591_amd import binding
    import workloads

    # the package has loaded the product library by now: swap in the instrumented one
    os.environ["DQ_LIBRARY_PATH"] = build.TIMELINE_LIB_PATH
    binding.lib = binding._load()
    lib = binding.lib

    dev = "cuda:0"
    if args.issue_probe:
        issue_probe(lib, torch, dev)
        return
    w = workloads.get_workload(args.workload)
    fmt, cache0, lens, _ = bench.build_cache(dq, torch, w, dev, bench._InProcess())
    if not dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads):
        raise SystemExit("the matrix-core kernel does not take this workload")
    caches = [cache0] + [cache0.clone() for _ in range(7)]
    q = torch.from_numpy(workloads.query(w)).to(dev)
    lens_d = torch.from_numpy(lens.astype(np.int32)).to(dev)
    max_seq = int(lens.max())
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, max_seq, dev)
    out = torch.empty_like(q)
    flags = dq.decode_flags(unit_map=args.unit_map)
    slots = int(lib.dq_debug_timeline_slots())
    max_waves = 1 << 16
    buf = torch.zeros((max_waves, slots), dtype=torch.int64, device=dev)
    lib.dq_debug_timeline.argtypes = [C.c_void_p]
    lib.dq_debug_timeline.restype = None
    for i in range(args.launches):
        dq.attn_decode(caches[i % 8], q, lens_d, max_seq, ws, out=out, flags=flags)
    lib.dq_debug_timeline(buf.data_ptr())
    dq.attn_decode(caches[args.launches % 8], q, lens_d, max_seq, ws, out=out, flags=flags)
    lib.dq_debug_timeline(None)
    torch.cuda.synchronize()
    t = buf.cpu().numpy()
    live = t[:, 0] != 0
    t = t[live].astype(np.float64)
    n_waves = t.shape[0]
    t0 = t[:, 0].min()
    us = (t - t0) / 100.0                                        # 100 MHz counter
    us[t == 0] = np.nan
    print("workload %s: %d waves stamped, launch %d of %d back to back" % (w.name, n_waves, args.launches + 1, args.launches + 1))
    names = ["wave entry", "first tile's arithmetic starts"] + ["tile %d starts" % (k + 1) for k in range(16)] + \
            ["last tile done", "wave exit (merge, output)"]
    print("| event | waves | min | p10 | median | p90 | max |  (microseconds after the first wave's entry)")
    print("|---|---|---|---|---|---|---|")
    for s in range(20):
        col = us[:, s]
        col = col[~np.isnan(col)]
        if col.size == 0:
            continue
        print("| %s | %d | %.2f | %.2f | %.2f | %.2f | %.2f |" % (names[s], col.size, col.min(), np.percentile(col, 10),
                                                                 np.median(col), np.percentile(col, 90), col.max()))
    durs = [[] for _ in range(16)]                               # duration of a wave's k-th tile, k < 15
    for row in us:
        starts = [x for x in row[2:18] if not np.isnan(x)]
        if len(starts) == 16:                                    # later tiles overwrote the last slot
            starts = starts[:15]
        else:
            starts = starts + [row[18]]
        for k in range(len(starts) - 1):
            durs[k].append(starts[k + 1] - starts[k])
    print("median tile durations (us):", ", ".join("%.2f" % np.median(d) for d in durs if d))
    print("p90 tile durations (us):", ", ".join("%.2f" % np.percentile(d, 90) for d in durs if d))
    # waves are stamped in workgroup order; workgroup g (launch order) sits on XCD g % 8
    nw = int(t[0, 20])
    xcd = (live.nonzero()[0] // nw) % 8
    span = us[:, 18] - us[:, 2]
    print("%d waves per workgroup; first tile to last tile, median by XCD (workgroup index mod 8): %s"
          % (nw, ", ".join("%.1f" % np.nanmedian(span[xcd == k]) for k in range(8))))
    print("wave exit, median by XCD: %s" % ", ".join("%.1f" % np.nanmedian(us[xcd == k, 19]) for k in range(8)))
    # how evenly a workgroup's waves finish their tiles (they merge only when the last one is done)
    wg = live.nonzero()[0] // nw
    done = us[:, 18]
    spread = np.array([done[wg == g].max() - done[wg == g].min() for g in np.unique(wg)])
    idle = np.array([(done[wg == g].max() - done[wg == g]).mean() for g in np.unique(wg)])
    print("last tile done, slowest minus fastest wave of a workgroup: median %.2f, p90 %.2f, max %.2f us; "
          "mean wait of a wave for its workgroup's slowest: %.2f us" % (np.median(spread), np.percentile(spread, 90), spread.max(), idle.mean()))
    wg_done = np.array([done[wg == g].max() for g in np.unique(wg)])
    print("workgroups' last tile done: min %.2f, median %.2f, max %.2f us" % (wg_done.min(), np.median(wg_done), wg_done.max()))
    print("launch: first entry to last exit %.2f us; median wave exit %.2f us" % (np.nanmax(us[:, 19]), np.nanmedian(us[:, 19])))


def issue_probe(lib, torch, dev, iters=20000):
    import ctypes as C
    lib.dq_debug_issue_probe.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.dq_debug_issue_probe.restype = C.c_int32
    sink = torch.zeros(16, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    kinds = [(0, "none"), (1, "v_mfma_f32_16x16x4_f32"), (2, "v_mfma_f32_16x16x16_f16"), (3, "v_mfma_i32_16x16x64_i8"),
             (4, "v_mfma_f64_16x16x4_f64")]
    print("| four matrix instructions of | alone, ns per loop body | with 16 fp32 FMAs | the FMAs alone | sum |  (one wave's loop body; four waves per SIMD)")
    print("|---|---|---|---|---|")
    times = {}
    for kind, _ in kinds:
        for fma in (0, 1):
            if kind == 0 and not fma:
                continue
            for rep in range(2):       # the first launch warms up
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                rc = lib.dq_debug_issue_probe(kind, fma, iters, sink.data_ptr(), stream)
                e1.record()
                torch.cuda.synchronize()
                if rc != 0:
                    raise SystemExit("dq_debug_issue_probe failed: %d" % rc)
            # four waves per SIMD share it: the SIMD's time per loop body of one wave
            times[kind, fma] = e0.elapsed_time(e1) * 1e6 / (4 * iters) / 4    # four bodies per trip, four waves per SIMD
    for kind, name in kinds[1:]:
        print("| %s | %.1f | %.1f | %.1f | %.1f |" % (name, times[kind, 0], times[kind, 1], times[0, 1], times[kind, 0] + times[0, 1]))


if __name__ == "__main__":
    main()
