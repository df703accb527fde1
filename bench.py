#!/usr/bin/env python3
"""Benchmark: decode-step attention over a DecoQuant-compressed KV cache on one MI355X.

One "step" is one dq_attn_decode call (the whole hot path: fold, code streaming, online
softmax, P.V, small-tensor epilogue, split merge) for one layer of the workload.  The cache is
already resident in HBM when the timed region starts; steps rotate over several distinct copies
of the layer's cache so that the 256 MB last-level cache cannot serve the stream.

Prints ONE JSON line: decode tokens/s per layer (= batch / time per step), the HBM roofline
fraction of the streaming kernel (HIP events around that kernel inside the timed loop), and the
CPU oracle timed on the host cores on a bounded sample of the same workload.
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

# HBM bytes per launch of the streaming kernel from the rocprofv3 FETCH_SIZE + WRITE_SIZE runs kept
# under profiles/ (counter values scaled by what the same counters read for the plain read kernel
# of known size).  None where no such run exists.
PROFILED_TRAFFIC_BYTES = {
    ("llama7b_4bit", "mfma"): (71822 + 64) * 1.9988 * 1024,
    ("llama7b_2bit", "mfma"): (164026 + 128) * 1.9994 * 1024,
    ("llama7b_8bit", "mfma"): (137581 + 64) * 1.9994 * 1024,
    ("llama13b_mixed", "mfma"): (152212 + 352) * 2.0150 * 1024,
    ("gqa_long", "mfma"): (287272 + 764) * 1.9997 * 1024,
    ("gqa8_long", "mfma"): (359155 + 256) * 1.9997 * 1024,
    ("opt_d64_4bit", "mfma"): (71851 + 64) * 1.9988 * 1024,
    ("llama7b_4bit_n3", "mfma"): (72852 + 64) * 1.9988 * 1024,
}


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
    fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, w.i3, w.levels)
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
    return {
        "value": w.batch / layer_s,
        "unit": "decode tokens/s per layer",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d of %d (sequence, kv head) pairs at full length, decode time scaled x%.1f; "
                  "oracle compression of the same pairs took %.2f s wall" % (len(pairs), len(all_pairs), scale, t_compress),
        "decode_wall_s_sample": t_decode,
    }


# --------------------------------------------------------------------------------------------
# GPU side
# --------------------------------------------------------------------------------------------
def build_cache(dq, torch, w, dev):
    """Host-generate the layer's K/V, upload, compress every block on the GPU."""
    fmt = dq.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, w.i3, w.levels)
    tb = w.block_tokens
    total = w.max_seq + w.append_tokens
    nb = -(-total // tb)
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, nb, dev)
    cws = dq.compress_workspace(fmt, w.batch, w.kv_heads, dev)
    lens = workloads.seq_lens(w)
    kd = torch.empty((w.batch, w.kv_heads, nb * tb, w.head_dim), dtype=torch.float16, device=dev)
    vd = torch.empty_like(kd)
    kd.zero_(); vd.zero_()
    for b in range(w.batch):
        n = int(lens[b])
        for h in range(w.kv_heads):
            k, v = workloads.kv_pair(w, b, h, n)
            kd[b, h, :n] = torch.from_numpy(k).to(dev)
            vd[b, h, :n] = torch.from_numpy(v).to(dev)
    if w.append_tokens:   # the appended rows follow the cached ones and are compressed with them
        for b in range(w.batch):
            n = int(lens[b])
            for h in range(w.kv_heads):
                k, v = workloads.appended_pair(w, b, h)
                kd[b, h, n:n + w.append_tokens] = torch.from_numpy(k).to(dev)
                vd[b, h, n:n + w.append_tokens] = torch.from_numpy(v).to(dev)
        lens = lens + w.append_tokens
    lens_d = torch.from_numpy(lens).to(dev)
    for blk in range(nb):
        idx = torch.full((w.batch,), blk, dtype=torch.int32, device=dev)
        n_valid = torch.clamp(lens_d - blk * tb, 0, tb).to(torch.int32)
        idx = torch.where(n_valid > 0, idx, torch.full_like(idx, -1))
        dq.compress_kv(cache, kd[:, :, blk * tb:(blk + 1) * tb].contiguous(),
                       vd[:, :, blk * tb:(blk + 1) * tb].contiguous(), idx, n_valid, cws)
    torch.cuda.synchronize()
    # time the companion step: compressing one new block (block_tokens rows) per (sequence, kv head)
    spare = dq.alloc_cache(fmt, w.batch, w.kv_heads, 1, dev)
    k_blk, v_blk = kd[:, :, :tb].contiguous(), vd[:, :, :tb].contiguous()
    zero_idx = torch.zeros(w.batch, dtype=torch.int32, device=dev)
    # (as a serving loop calls it: the fp32 large tensors are not read back)
    for _ in range(3):
        dq.compress_kv(spare, k_blk, v_blk, zero_idx, None, cws, keep_large=False)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dq.compress_kv(spare, k_blk, v_blk, zero_idx, None, cws, keep_large=False)
    e1.record()
    torch.cuda.synchronize()
    compress_ms = e0.elapsed_time(e1) / 10
    del kd, vd, spare
    return fmt, cache, lens, compress_ms


def algorithmic_bytes(w, lens) -> float:
    """Bytes the method itself must read per step: codes + steps + small tensors of every cached
    token of every kv head (keys and values), plus q and out."""
    small = 2 * w.j1 * w.j1 + (2 * w.i3 * w.i3 if w.i3 > 1 else 0)     # bytes of fp16 small tensors per block
    per_tok = 2 * (w.head_dim * w.bits / 8 + 2 * w.head_dim / w.group) + 2 * small / w.block_tokens
    toks = float(np.sum(lens.astype(np.int64))) * w.kv_heads
    return per_tok * toks + w.batch * w.q_heads * w.head_dim * 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=2000,
                    help="untimed steps first; the GPU clocks take tens of milliseconds of load to settle")
    ap.add_argument("--workload", default="llama7b_4bit", choices=sorted(workloads.WORKLOADS))
    ap.add_argument("--layers", type=int, default=8, help="distinct cache copies the steps rotate over")
    ap.add_argument("--cpu-pairs", type=int, default=256, help="(sequence, head) pairs the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--generic", action="store_true", help="force the reference-grade HIP kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only (this build has no multi-GPU path); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    w = workloads.get_workload(args.workload)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args.workload, args.cpu_pairs)   # before any GPU initialisation (fork)

    import torch
    import paper_2405_12591_amd as dq
    dev = "cuda:0"
    torch.cuda.set_device(0)
    fmt, cache0, lens, compress_ms = build_cache(dq, torch, w, dev)
    n_layers = max(1, args.layers)
    caches = [cache0] + [cache0.clone() for _ in range(n_layers - 1)]
    q = torch.from_numpy(workloads.query(w)).to(dev)
    lens_d = torch.from_numpy(lens).to(dev)
    max_seq = int(lens.max())
    ws = dq.decode_workspace(fmt, w.batch, w.q_heads, w.kv_heads, max_seq, dev)
    out = torch.empty_like(q)
    flags = dq.DECODE_FORCE_GENERIC if args.generic else dq.DECODE_AUTO
    path = "generic" if (args.generic or not dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)) else "mfma"

    K, W = args.steps, args.warmup
    kev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    for a, b in kev:   # record once so that the handles exist
        a.record(); b.record()
    torch.cuda.synchronize()

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
    total_ms = t_start.elapsed_time(t_stop)
    ms_per_step = total_ms / K
    # the same K steps again with a HIP event pair around each streaming kernel (its duration
    # for the roofline); the event records lengthen the gaps between kernels, not the kernels
    t_start.record()
    for i in range(K):
        dq.attn_decode(caches[i % n_layers], q, lens_d, max_seq, ws, out=out, flags=flags, kernel_events=kev[i])
    t_stop.record()
    torch.cuda.synchronize()
    ms_per_step_with_events = t_start.elapsed_time(t_stop) / K
    kernel_ms = np.array([a.elapsed_time(b) for a, b in kev])

    # read-bandwidth ceiling: plain 128-bit loads over the same cache bytes
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    big = [c.t["k_codes"] for c in caches] + [c.t["v_codes"] for c in caches]
    for t in big[:4]:
        dq.stream_read(t, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in big:
        dq.stream_read(t, sink)
    e1.record()
    torch.cuda.synchronize()
    stream_gbps = sum(t.numel() for t in big) / (e0.elapsed_time(e1) * 1e-3) / 1e9

    alg = algorithmic_bytes(w, lens)
    achieved = alg / (kernel_ms.mean() * 1e-3) / 1e9
    result = {
        "metric": "decode-attention tokens/s per layer, 4-bit DecoQuant KV cache" if w.bits == 4 else
                  "decode-attention tokens/s per layer, %d-bit DecoQuant KV cache" % w.bits,
        "value": w.batch / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("u%d codes on int8 MFMA, f32 accumulate" if path == "mfma" else "u%d codes, f32") % w.bits,
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.q_heads, "kv_heads": w.kv_heads,
                   "head_dim": w.head_dim, "seq_len": [int(lens.min()), int(lens.max())], "bits": w.bits,
                   "group": w.group, "block_tokens": w.block_tokens, "j1": w.j1, "local_tensors": 3 if w.i3 > 1 else 2,
                   "kernel_path": path,
                   "cache_copies_rotated": n_layers, "cache_bytes_per_layer": cache0.nbytes()},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": PROFILED_TRAFFIC_BYTES.get((w.name, path)),
                     "kernel_ms_mean": float(kernel_ms.mean()), "kernel_ms_median": float(np.median(kernel_ms)),
                     "algorithmic_bytes_per_launch": alg},
        "cpu_baseline": cpu,
        "kv_tokens_streamed_per_s": float(np.sum(lens.astype(np.int64))) * w.kv_heads / (ms_per_step * 1e-3),
        "whole_call_GBps": alg / (ms_per_step * 1e-3) / 1e9,
        "stream_read_ceiling_GBps": stream_gbps,
        "frac_of_stream_read_ceiling": achieved / stream_gbps if stream_gbps > 0 else None,
        "compress_kv": {"ms_per_call": compress_ms, "blocks_per_call": 2 * w.batch * w.kv_heads,
                        "rows_per_block": w.block_tokens},
        "host_wall_s_timed_region": wall,
        "ms_per_step_with_kernel_events": ms_per_step_with_events,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
