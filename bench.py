#!/usr/bin/env python3
"""Benchmark: decode-step attention over a DecoQuant-compressed KV cache on one MI355X.

One "step" is one dq_attn_decode call (the whole hot path: fold, code streaming, online
softmax, P.V, small-tensor epilogue, split merge) for one layer of the workload.  The cache is
already resident in HBM when the timed region starts; steps rotate over several distinct copies
of the layer's cache so that the 256 MB last-level cache cannot serve the stream.

Prints ONE JSON line.  Its top-level fields describe the headline workload (the largest of the
single-GPU configurations, `gqa_long`): decode tokens/s per layer (= batch / time per step), the
HBM roofline fraction of the streaming kernel (HIP events around that kernel inside a second pass
of the same steps), and the CPU oracle timed on the host cores on a bounded sample of the same
workload.  `per_config` carries the same figures for every large configuration (7B 4-bit, 7B 2-bit,
13B mixed lengths with its compression of 128 appended rows, long-context GQA), and every entry
times the companion step `compress_kv` (one new block per sequence and head) and the prompt
compression (`compress_kv_blocks`) that built its cache.
"""
from __future__ import annotations

import argparse
import json
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads  # noqa: E402

HBM_PEAK_GBPS = 8000.0
FP64_MFMA_PEAK_TFLOPS = 78.6
# the large single-GPU configurations, smallest to largest; the last one carries the headline
LARGE_CONFIGS = ["llama7b_4bit", "llama7b_2bit", "llama13b_mixed", "gqa_long"]

# HBM bytes per launch of the streaming kernel from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs kept
# under profiles/ (counter values in KiB; FETCH_SIZE scaled by what it reads for the plain read kernel
# of known size, WRITE_SIZE as it is: it reads 1.0 x a known write).  A constant of the profiled build, not a quantity of this run: the run
# cannot host the profiler.  None where no such run exists.
PROFILED_TRAFFIC_BYTES = {
    ("llama7b_4bit", "mfma"): (71814.0 * 1.9994 + 64.0) * 1024,
    ("llama7b_2bit", "mfma"): (164017.5 * 1.9997 + 128.0) * 1024,
    ("llama7b_8bit", "mfma"): (137574.3 * 1.9997 + 64.0) * 1024,
    ("llama13b_mixed", "mfma"): (152201.9 * 1.9998 + 352.5) * 1024,
    ("gqa_long", "mfma"): (287280.5 * 1.9999 + 764.0) * 1024,
    ("gqa8_long", "mfma"): (353847.3 * 1.9999 + 256.0) * 1024,
    ("opt_d64_4bit", "mfma"): (71839.5 * 1.9994 + 64.0) * 1024,
    ("llama7b_4bit_n3", "mfma"): (72855.0 * 1.9994 + 64.0) * 1024,
}
TRAFFIC_SOURCE = ("profiles/decode_mfma_llama7b_4bit.md, profiles/decode_mfma_other_workloads.md: rocprofv3 --pmc "
                  "FETCH_SIZE (scaled by the read-kernel calibration) + WRITE_SIZE per launch (a constant of the "
                  "profiled build, not measured in this run)")


# --------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, forked workers, before the GPU is initialised
# --------------------------------------------------------------------------------------------
def _cpu_worker(rank, n_workers, wname, pairs, barrier, queue):
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass
    from oracle import decoquant_oracle as O
    w = workloads.get_workload(wname)
    fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, w.i3, w.levels, w.i1)
    mine = pairs[rank::n_workers]
    lens = workloads.seq_lens(w)
    q = workloads.query(w)
    rep = w.q_heads // w.kv_heads
    caches = []
    t0 = time.perf_counter()
    if w.append_tokens:
        lens = lens + w.append_tokens
    for b, h in mine:
        n = int(lens[b])
        k, v = workloads.kv_pair(w, b, h, n - w.append_tokens)
        if w.append_tokens:
            ka, va = workloads.appended_pair(w, b, h)
            k, v = np.concatenate([k, ka]), np.concatenate([v, va])
        c = O.empty_cache(fmt, 1, 1, -(-n // w.block_tokens))
        O.compress_sequence(c, fmt, 0, 0, k, v)
        caches.append(c)
    t_compress = time.perf_counter() - t0
    barrier.wait()
    t0 = time.perf_counter()
    for (b, h), c in zip(mine, caches):
        qq = q[b:b + 1, h * rep:(h + 1) * rep]
        O.attention_decode(c, fmt, qq, lens[b:b + 1])
    t_decode = time.perf_counter() - t0
    queue.put((rank, t_compress, t_decode))


def cpu_baseline(wname: str, n_pairs: int):
    w = workloads.get_workload(wname)
    all_pairs = [(b, h) for b in range(w.batch) for h in range(w.kv_heads)]
    stride = max(1, len(all_pairs) // n_pairs)
    pairs = all_pairs[::stride][:n_pairs]
    cores = min(os.cpu_count() or 1, 16, len(pairs))
    ctx = mp.get_context("fork")
    barrier = ctx.Barrier(cores)
    queue = ctx.Queue()
    procs = [ctx.Process(target=_cpu_worker, args=(r, cores, wname, pairs, barrier, queue)) for r in range(cores)]
    for p in procs:
        p.start()
    res = [queue.get() for _ in procs]
    for p in procs:
        p.join()
    t_decode = max(r[2] for r in res)     # wall time of the decode phase (workers start it together)
    t_compress = max(r[1] for r in res)
    scale = len(all_pairs) / len(pairs)
    layer_s = t_decode * scale
    blocks = sum(2 * -(-int((workloads.seq_lens(w) + w.append_tokens)[b]) // w.block_tokens) for b, _ in pairs)
    return {
        "value": w.batch / layer_s,
        "unit": "decode tokens/s per layer",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d of %d (sequence, kv head) pairs at full length, decode time scaled x%.1f; "
                  "oracle compression of the same pairs (%d blocks) took %.2f s wall"
                  % (len(pairs), len(all_pairs), scale, blocks, t_compress),
        "decode_wall_s_sample": t_decode,
        "compress_blocks_per_s": blocks / t_compress if t_compress > 0 else None,
    }


# --------------------------------------------------------------------------------------------
# Input generation on the host cores (forked before the GPU is initialised; draws only)
# --------------------------------------------------------------------------------------------
def _gen_pair(task):
    wname, b, h, n = task
    w = workloads.get_workload(wname)
    k, v = workloads.kv_pair(w, b, h, n)
    if w.append_tokens:
        ka, va = workloads.appended_pair(w, b, h)
        k, v = np.concatenate([k, ka]), np.concatenate([v, va])
    return b, h, k, v


class _InProcess:
    """Stand-in for the worker pool: draws the inputs in the calling process."""

    def imap_unordered(self, fn, tasks, chunksize=1):
        return map(fn, tasks)

    def close(self):
        pass

    def join(self):
        pass


# --------------------------------------------------------------------------------------------
# GPU side
# --------------------------------------------------------------------------------------------
def block_bytes(w):
    """Algorithmic bytes of compressing one block: its fp16 rows in; codes, steps and the small
    tensor(s) out."""
    tb, d = w.block_tokens, w.head_dim
    small = 2 * w.j1 * w.j1 + (2 * w.i3 * w.i3 if w.i3 > 1 else 0)
    return tb * d * 2, tb * d * w.bits // 8 + tb * (d // w.group) * 2 + small


def block_flops(w):
    """fp64 flops of one block's decomposition as the library does it: Gram matrix (j1 x j1 over
    T_b*j2 columns), projection (the same count), and the Jacobi iteration (about six sweeps of
    j1*(j1-1)/2 rotations over two j1 x j1 matrices, 12 flops per rotated pair of entries)."""
    cols = w.block_tokens * w.j2
    return 2 * 2 * w.j1 * w.j1 * cols + 6 * (w.j1 * (w.j1 - 1) // 2) * 2 * w.j1 * 12


def build_cache(dq, torch, w, dev, pool):
    """Host-generate the layer's K/V, upload, compress the whole prompt with one
    dq_compress_kv_blocks call (timed), then time the companion step: compressing one new block
    per (sequence, kv head)."""
    fmt = dq.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, w.i3, w.levels, w.i1)
    tb = w.block_tokens
    total = w.max_seq + w.append_tokens
    nb = -(-total // tb)
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, dev)
    lens = workloads.seq_lens(w)
    kd = torch.zeros((w.batch, w.kv_heads, nb * tb, w.head_dim), dtype=torch.float16, device=dev)
    vd = torch.zeros_like(kd)
    tasks = [(w.name, b, h, int(lens[b])) for b in range(w.batch) for h in range(w.kv_heads)]
    t0 = time.perf_counter()
    for b, h, k, v in pool.imap_unordered(_gen_pair, tasks, chunksize=1):
        kd[b, h, :k.shape[0]] = torch.from_numpy(k).to(dev)
        vd[b, h, :v.shape[0]] = torch.from_numpy(v).to(dev)
    gen_s = time.perf_counter() - t0
    lens = lens + w.append_tokens     # the appended rows follow the cached ones and are compressed with them
    lens_d = torch.from_numpy(lens.astype(np.int32)).to(dev)
    first = torch.zeros(w.batch, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pws = dq.compress_workspace(fmt, w.batch, w.kv_heads, dev, t_new=nb * tb)
    n_rep = 3
    for i in range(1 + n_rep):        # the first call warms up; every call writes the same cache
        if i == 1:
            e0.record()
        dq.compress_kv_blocks(cache, kd, vd, first, lens_d, pws, keep_large=False)
    e1.record()
    torch.cuda.synchronize()
    prefill_ms = e0.elapsed_time(e1) / n_rep
    status = int(pws[:4].view(torch.int32).item())
    del pws
    prefill_blocks = int(sum(2 * w.kv_heads * -(-int(n) // tb) for n in lens))
    # the companion step: one new block (block_tokens rows) per (sequence, kv head), as a serving loop
    # calls it (the fp32 large tensors are not read back); for the workload that appends rows these
    # are the appended rows
    spare = dq.alloc_cache(fmt, w.batch, w.kv_heads, 1, dev)
    cws = dq.compress_workspace(fmt, w.batch, w.kv_heads, dev)
    if w.append_tokens:
        rows = torch.stack([kd[b, :, int(lens[b]) - tb:int(lens[b])] for b in range(w.batch)]).contiguous(), \
               torch.stack([vd[b, :, int(lens[b]) - tb:int(lens[b])] for b in range(w.batch)]).contiguous()
    else:
        rows = kd[:, :, :tb].contiguous(), vd[:, :, :tb].contiguous()
    zero_idx = torch.zeros(w.batch, dtype=torch.int32, device=dev)
    for _ in range(20):
        dq.compress_kv(spare, rows[0], rows[1], zero_idx, None, cws, keep_large=False)
    e0.record()
    for _ in range(50):
        dq.compress_kv(spare, rows[0], rows[1], zero_idx, None, cws, keep_large=False)
    e1.record()
    torch.cuda.synchronize()
    compress_ms = e0.elapsed_time(e1) / 50
    del kd, vd, spare, cws
    n_blk = 2 * w.batch * w.kv_heads
    b_in, b_out = block_bytes(w)
    comp = {
        "ms_per_call": compress_ms, "blocks_per_call": n_blk, "rows_per_block": tb,
        "ns_per_block": compress_ms * 1e6 / n_blk,
        "roofline": {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBPS,
                     "achieved": n_blk * (b_in + b_out) / (compress_ms * 1e-3) / 1e9,
                     "frac": n_blk * (b_in + b_out) / (compress_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_block": b_in + b_out,
                     "fp64_tflops": n_blk * block_flops(w) / (compress_ms * 1e-3) / 1e12,
                     "fp64_frac_of_mfma_peak": n_blk * block_flops(w) / (compress_ms * 1e-3) / 1e12 / FP64_MFMA_PEAK_TFLOPS,
                     "note": "a call of a few hundred blocks is bound by the latency of one block's chain "
                             "(Gram matrix, Jacobi iteration, projection, quantizer), not by either roof"},
        "prefill": {"ms_per_call": prefill_ms, "blocks_per_call": prefill_blocks,
                    "ns_per_block": prefill_ms * 1e6 / prefill_blocks,
                    "achieved_GBps": prefill_blocks * (b_in + b_out) / (prefill_ms * 1e-3) / 1e9,
                    "frac_of_hbm_peak": prefill_blocks * (b_in + b_out) / (prefill_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                    "status_word": status},
        "host_generation_s": gen_s,
    }
    return fmt, cache, lens, comp


def algorithmic_bytes(w, lens) -> float:
    """Bytes the method itself must read per step: codes + steps + small tensors of every cached
    token of every kv head (keys and values), plus q and out."""
    small = 2 * w.j1 * w.j1 + (2 * w.i3 * w.i3 if w.i3 > 1 else 0)     # bytes of fp16 small tensors per block
    per_tok = 2 * (w.head_dim * w.bits / 8 + 2 * w.head_dim / w.group) + 2 * small / w.block_tokens
    toks = float(np.sum(lens.astype(np.int64))) * w.kv_heads
    return per_tok * toks + w.batch * w.q_heads * w.head_dim * 4


def settle_clocks(dq, torch, caches, q, lens_d, max_seq, ws, out, flags, ms=150.0):
    """The GPU clocks take tens of milliseconds of load to settle: keep the device busy with the very
    calls that will be timed (untimed here) before the warm-up steps."""
    n_layers = len(caches)
    t0 = time.perf_counter()
    i = 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(50):
            dq.attn_decode(caches[i % n_layers], q, lens_d, max_seq, ws, out=out, flags=flags)
            i += 1
        torch.cuda.synchronize()
    return i


def run_config(dq, torch, w, K, W, n_layers, generic, pool, dev="cuda:0", shape_tag=None, launch=(0, 0)):
    fmt, cache0, lens, comp = build_cache(dq, torch, w, dev, pool)
    caches = [cache0] + [cache0.clone() for _ in range(n_layers - 1)]
    q = torch.from_numpy(workloads.query(w)).to(dev)
    lens_d = torch.from_numpy(lens.astype(np.int32)).to(dev)
    max_seq = int(lens.max())
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, max_seq, dev)
    out = torch.empty_like(q)
    flags = (dq.DECODE_FORCE_GENERIC if generic else dq.DECODE_AUTO) | dq.decode_flags(splits=launch[0], waves=launch[1])
    path = "generic" if (generic or not dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)) else "mfma"

    kev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    for a, b in kev:   # record once so that the handles exist
        a.record(); b.record()
    torch.cuda.synchronize()
    settled = settle_clocks(dq, torch, caches, q, lens_d, max_seq, ws, out, flags)

    for i in range(W):
        dq.attn_decode(caches[i % n_layers], q, lens_d, max_seq, ws, out=out, flags=flags)
    torch.cuda.synchronize()
    # timed region: exactly K steps back to back on the stream
    t_start, t_stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    t_start.record()
    for i in range(K):
        dq.attn_decode(caches[i % n_layers], q, lens_d, max_seq, ws, out=out, flags=flags)
    t_stop.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_per_step = t_start.elapsed_time(t_stop) / K
    # the same K steps again with a HIP event pair around each streaming kernel (its duration
    # for the roofline); the event records lengthen the gaps between kernels, not the kernels
    t_start.record()
    for i in range(K):
        dq.attn_decode(caches[i % n_layers], q, lens_d, max_seq, ws, out=out, flags=flags, kernel_events=kev[i])
    t_stop.record()
    torch.cuda.synchronize()
    ms_per_step_with_events = t_start.elapsed_time(t_stop) / K
    kernel_ms = np.array([a.elapsed_time(b) for a, b in kev])

    # plain read of the same number of bytes (one buffer per rotation slot, each as large as the
    # cache, sixteen 1 KB loads in flight per wave): what a kernel that only streams reaches
    nbytes = cache0.nbytes() // 4096 * 4096
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(max(2, min(n_layers, 4)))]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    for i in range(40):
        dq.stream_read(bufs[i % len(bufs)], sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(40):
        dq.stream_read(bufs[i % len(bufs)], sink)
    e1.record()
    torch.cuda.synchronize()
    stream_gbps = 40 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del bufs

    alg = algorithmic_bytes(w, lens)
    achieved = alg / (kernel_ms.mean() * 1e-3) / 1e9
    res = {
        "workload": w.name + (shape_tag or ""),
        "value": w.batch / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "steps": K, "warmup": W, "clock_settle_steps_before_warmup": settled,
        "ms_per_step": ms_per_step,
        "dtype": ("u%d codes on int8 MFMA, f32 accumulate" if path == "mfma" else "u%d codes, f32") % w.bits,
        "config": {"workload": w.name + (shape_tag or ""), "batch": w.batch, "q_heads": w.q_heads, "kv_heads": w.kv_heads,
                   "head_dim": w.head_dim, "seq_len": [int(lens.min()), int(lens.max())], "bits": w.bits,
                   "group": w.group, "block_tokens": w.block_tokens, "j1": w.j1, "local_tensors": 3 if w.i3 > 1 else 2,
                   "kernel_path": path, "launch_override": list(launch) if any(launch) else None,
                   "cache_copies_rotated": n_layers, "cache_bytes_per_layer": cache0.nbytes()},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None if shape_tag else PROFILED_TRAFFIC_BYTES.get((w.name, path)),
                     "traffic_source": TRAFFIC_SOURCE,
                     "kernel_ms_mean": float(kernel_ms.mean()), "kernel_ms_median": float(np.median(kernel_ms)),
                     "algorithmic_bytes_per_launch": alg},
        "kv_tokens_streamed_per_s": float(np.sum(lens.astype(np.int64))) * w.kv_heads / (ms_per_step * 1e-3),
        "whole_call_GBps": alg / (ms_per_step * 1e-3) / 1e9,
        "stream_read_GBps": stream_gbps,
        "compress_kv": comp,
        "host_wall_s_timed_region": wall,
        "ms_per_step_with_kernel_events": ms_per_step_with_events,
    }
    del caches, cache0, ws
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=500, help="untimed steps ahead of the timed ones")
    ap.add_argument("--workload", default="gqa_long", choices=sorted(workloads.WORKLOADS),
                    help="the headline workload (top-level fields of the line)")
    ap.add_argument("--only", action="store_true", help="measure the headline workload alone (no per_config list)")
    ap.add_argument("--layers", type=int, default=8, help="distinct cache copies the steps rotate over")
    ap.add_argument("--cpu-pairs", type=int, default=32,
                    help="(sequence, head) pairs the CPU oracle is timed on for the headline workload "
                         "(half as many for the other entries of per_config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-workers", type=int, default=16,
                    help="host processes that draw the synthetic inputs (0: in this process, for runs under a profiler)")
    ap.add_argument("--generic", action="store_true", help="force the reference-grade HIP kernel")
    ap.add_argument("--launch", default=None, metavar="SPLITS,WAVES",
                    help="with --only: override the library's launch shape of the matrix-core kernel (workgroups per "
                         "(sequence, kv head); waves per workgroup, 4 or 8; 0 leaves either to the library)")
    ap.add_argument("--shape", default=None, metavar="B,HQ,HKV,S",
                    help="with --only: the workload's format and value distribution on another shape (batch, query "
                         "heads, kv heads, tokens per sequence); no CPU baseline and no profiled traffic for such a run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only (this build has no multi-GPU path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    shaped = None
    if args.shape:
        if not args.only:
            print("--shape needs --only", file=sys.stderr)
            sys.exit(2)
        import dataclasses
        b_, hq_, hkv_, s_ = (int(x) for x in args.shape.split(","))
        base = workloads.get_workload(args.workload)
        if b_ < 1 or hkv_ < 1 or hq_ % hkv_ or s_ < base.block_tokens or s_ % base.block_tokens or base.append_tokens:
            print("--shape: B,HQ,HKV,S with HQ a multiple of HKV and S a multiple of the block size; not for workloads "
                  "that append rows", file=sys.stderr)
            sys.exit(2)
        shaped = dataclasses.replace(base, batch=b_, q_heads=hq_, kv_heads=hkv_, max_seq=s_, min_seq=s_)
        args.no_cpu_baseline = True
    names = [args.workload] if args.only else [n for n in LARGE_CONFIGS if n != args.workload] + [args.workload]
    cpu = {}
    if not args.no_cpu_baseline:      # before any GPU initialisation (fork)
        for n in names:
            cpu[n] = cpu_baseline(n, args.cpu_pairs if n == args.workload else max(1, args.cpu_pairs // 2))
    # workers that draw the synthetic inputs (forked before the GPU is initialised; they never touch it)
    pool = mp.get_context("fork").Pool(min(os.cpu_count() or 1, args.gen_workers)) if args.gen_workers > 0 else _InProcess()

    import torch
    import paper_2405_12591_amd as dq
    if not torch.cuda.is_available():
        print("bench.py needs a GPU: there is no CPU path", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup
    n_layers = max(1, args.layers)
    results = {}
    for n in names:
        w = shaped or workloads.get_workload(n)
        results[n] = run_config(dq, torch, w, K, W, n_layers, args.generic, pool,
                                shape_tag=("@" + args.shape) if shaped else None,
                                launch=tuple(int(x) for x in args.launch.split(",")) if (args.launch and args.only) else (0, 0))
        results[n]["cpu_baseline"] = cpu.get(n)
    pool.close()
    pool.join()

    head = results[args.workload]
    w = shaped or workloads.get_workload(args.workload)
    line = {
        "metric": "decode-attention tokens/s per layer, 4-bit DecoQuant KV cache" if w.bits == 4 else
                  "decode-attention tokens/s per layer, %d-bit DecoQuant KV cache" % w.bits,
        "value": head["value"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": head["config"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
    }
    for key in ("kv_tokens_streamed_per_s", "whole_call_GBps", "stream_read_GBps", "compress_kv",
                "clock_settle_steps_before_warmup", "host_wall_s_timed_region", "ms_per_step_with_kernel_events"):
        line[key] = head[key]
    if not args.only:
        line["per_config"] = [results[n] for n in LARGE_CONFIGS if n in results]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
