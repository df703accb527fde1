"""Seeded random sweep of the decode entry points against the oracle: code widths, group sizes,
head groupings, block sizes, ragged lengths (0, 1, around a tile edge, full), fp16 tails of every
length and capacity, and forced launch shapes (splits per sequence, waves per workgroup), so that
every tail mode and merge path of the matrix-core kernel and the plain kernel is exercised; and of
the compression entry point against the oracle's properties and against itself (with and without
the fp32 rows kept, every wave count).  `--sweep-scale N` runs N times as many seeds of the two
wide sweeps (`pytest tests/test_gpu_sweep.py -m gpu -s --sweep-scale 40` prints every case and the
worst error of each seed as a fraction of the tolerance)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, oracle_cache_for_pairs, tolerance

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,i3", [(11, 1), (12, 1), (13, 1), (21, 8), (22, 8), (23, 8)])
def test_random_decode_cases(seed, i3):
    """i3 = 8: the same sweep over caches in the three-tensor form."""
    rng = np.random.default_rng(seed)
    for case in range(16):
        bits = int(rng.choice([2, 4, 8]))
        group = int(rng.choice([64, 128]))
        rep = int(rng.choice([1, 2, 4, 8, 3, 7] if group == 128 else [1, 2, 4, 3]))
        kvh, batch = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 3]))
        tb = int(rng.choice([128, 256]))
        max_seq = int(rng.choice([128, 300, 640, 1100, 2100]))
        w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh * rep, kv_heads=kvh,
                                max_seq=-(-max_seq // tb) * tb, min_seq=-(-max_seq // tb) * tb, bits=bits, group=group,
                                block_tokens=tb, seed=3000 + 100 * seed + case, i3=i3)
        fmt, ofmt = formats(w)
        lens = np.array([int(rng.choice([0, 1, 127, 128, 129, max_seq, int(rng.integers(0, max_seq + 1))]))
                         for _ in range(batch)], np.int32)
        lens = np.minimum(lens, max_seq)
        use_tail = bool(rng.integers(0, 2))
        cap = int(rng.choice([16, 128, 256]))
        tl = np.array([int(rng.choice([0, 1, cap, int(rng.integers(0, cap + 1))])) for _ in range(batch)], np.int32)
        splits, waves = str(rng.choice(["", "1", "2", "3", "5"])), str(rng.choice(["", "4", "8"]))
        shape = dq.decode_flags(splits=int(splits or 0), waves=int(waves or 0))   # launch-shape overrides in the flags word
        print("seed %d i3=%d case %d: bits=%d G=%d rep=%d kvh=%d B=%d Tb=%d max_seq=%d lens=%s tail=%s cap=%d tl=%s splits=%r waves=%r"
              % (seed, i3, case, bits, group, rep, kvh, batch, tb, max_seq, lens.tolist(), use_tail, cap, tl.tolist(), splits, waves),
              flush=True)
        pairs = [(b, h) for b in range(batch) for h in range(kvh)]
        cache = oracle_cache_for_pairs(w, ofmt, pairs, lens, seed=case)
        q = workloads.query(w)
        kt = (rng.standard_normal((batch, kvh, cap, 128)) * 2).astype(np.float16)
        vt = (rng.standard_normal((batch, kvh, cap, 128)) * 2).astype(np.float16)
        for b in range(batch):            # rows beyond the tail length may hold anything
            kt[b, :, tl[b]:] = np.float16(np.nan)
            vt[b, :, tl[b]:] = np.float16(np.inf)
        if use_tail:
            want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
        else:
            want = O.attention_decode(cache, ofmt, q, lens)
        dcache = dq.cache_from_numpy(fmt, cache, DEV)
        ws = dq.decode_workspace(fmt, batch, w.q_heads, kvh, max_seq, DEV)
        qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
        tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV)) if use_tail else None
        o32 = torch.empty((batch, w.q_heads, 128), dtype=torch.float32, device=DEV)
        for flags in (dq.DECODE_AUTO, dq.DECODE_FORCE_GENERIC):
            out = dq.attn_decode(dcache, qd, ld, max_seq, ws, out_f32=o32, flags=flags | shape, tail=tail)
            again = dq.attn_decode(dcache, qd, ld, max_seq, ws, flags=flags | shape, tail=tail)   # counters left clean
            torch.cuda.synchronize()
            g16, g32 = out.cpu().numpy().astype(np.float64), o32.cpu().numpy().astype(np.float64)
            assert torch.equal(out, again), (seed, case, flags)
            assert (np.abs(g16 - want) <= tolerance(want)).all(), (seed, case, flags, np.nanmax(np.abs(g16 - want)))
            assert (np.abs(g32 - want) <= np.maximum(2e-3, 1e-4 * np.abs(want))).all(), (seed, case, flags)


def test_random_decode_cases_wide(sweep_seed):
    """The same comparison over more of the format space: both level sets, heads of 64 channels (pairs
    on the matrix-core path), two and three local tensors, the value distributions of all workloads."""
    rng = np.random.default_rng(1000 + sweep_seed)
    worst = 0.0
    for case in range(16):
        bits, group = int(rng.choice([2, 4, 8])), int(rng.choice([64, 128]))
        rep = int(rng.choice([1, 2, 4, 8, 3, 7, 5] if group == 128 else [1, 2, 4, 3]))
        i3, levels = int(rng.choice([1, 8])), int(rng.choice([0, 1]))
        d64 = bool(rng.integers(0, 4) == 0)
        kvh, batch = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 3]))
        if d64:
            group, rep, i3, kvh = 64, 1, int(rng.choice([1, 1, 8])), int(rng.choice([2, 3, 4]))
        d = 64 if d64 else 128
        tb = int(rng.choice([128, 256]))
        max_seq = int(rng.choice([128, 300, 640, 1100, 2100]))
        base = str(rng.choice(["llama7b_4bit", "llama13b_mixed", "gqa_long", "plain"]))
        bw = workloads.get_workload("llama7b_4bit" if base == "plain" else base)
        if base == "plain":
            bw = dataclasses.replace(bw, dist="normal", n_outlier=2)
        w = dataclasses.replace(bw, head_dim=d, j1=d // 8, j2=8, levels=levels, n_outlier=min(bw.n_outlier, 4),
                                append_tokens=0, batch=batch, q_heads=kvh * rep, kv_heads=kvh,
                                max_seq=-(-max_seq // tb) * tb, min_seq=-(-max_seq // tb) * tb, bits=bits, group=group,
                                block_tokens=tb, seed=20000 + 100 * sweep_seed + case, i3=i3)
        fmt, ofmt = formats(w)
        lens = np.array([int(rng.choice([0, 1, 127, 128, 129, max_seq, int(rng.integers(0, max_seq + 1))]))
                         for _ in range(batch)], np.int32)
        lens = np.minimum(lens, max_seq)
        use_tail = bool(rng.integers(0, 2))
        cap = int(rng.choice([16, 128, 256]))
        tl = np.array([int(rng.choice([0, 1, cap, int(rng.integers(0, cap + 1))])) for _ in range(batch)], np.int32)
        splits, waves = int(rng.choice([0, 1, 2, 3, 5])), int(rng.choice([0, 4, 8]))
        shape = dq.decode_flags(splits=splits, waves=waves)
        print("wide seed %d case %d: %s d=%d levels=%d i3=%d bits=%d G=%d rep=%d kvh=%d B=%d Tb=%d max_seq=%d lens=%s tail=%s cap=%d "
              "tl=%s splits=%d waves=%d" % (sweep_seed, case, base, d, levels, i3, bits, group, rep, kvh, batch, tb, max_seq,
                                            lens.tolist(), use_tail, cap, tl.tolist(), splits, waves), flush=True)
        pairs = [(b, h) for b in range(batch) for h in range(kvh)]
        cache = oracle_cache_for_pairs(w, ofmt, pairs, lens, seed=case)
        q = workloads.query(w)
        kt = (rng.standard_normal((batch, kvh, cap, d)) * 2).astype(np.float16)
        vt = (rng.standard_normal((batch, kvh, cap, d)) * 2).astype(np.float16)
        for b in range(batch):
            kt[b, :, tl[b]:] = np.float16(np.nan)
            vt[b, :, tl[b]:] = np.float16(np.inf)
        if use_tail:
            want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
        else:
            want = O.attention_decode(cache, ofmt, q, lens)
        dcache = dq.cache_from_numpy(fmt, cache, DEV)
        ws = dq.decode_workspace(fmt, batch, w.q_heads, kvh, max_seq, DEV)
        qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
        tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV)) if use_tail else None
        o32 = torch.empty((batch, w.q_heads, d), dtype=torch.float32, device=DEV)
        for flags in (dq.DECODE_AUTO, dq.DECODE_FORCE_GENERIC):
            out = dq.attn_decode(dcache, qd, ld, max_seq, ws, out_f32=o32, flags=flags | shape, tail=tail)
            again = dq.attn_decode(dcache, qd, ld, max_seq, ws, flags=flags | shape, tail=tail)
            torch.cuda.synchronize()
            g16, g32 = out.cpu().numpy().astype(np.float64), o32.cpu().numpy().astype(np.float64)
            assert torch.equal(out, again), (sweep_seed, case, flags)
            r16 = float(np.max(np.abs(g16 - want) / tolerance(want)))
            r32 = float(np.max(np.abs(g32 - want) / np.maximum(2e-3, 1e-4 * np.abs(want))))
            assert r16 <= 1.0 and r32 <= 1.0, (sweep_seed, case, flags, r16, r32)   # (a NaN fails too)
            worst = max(worst, r16, r32)
    print("wide seed %d: 16 cases, worst error / tolerance %.3f" % (sweep_seed, worst), flush=True)


def test_random_compress_cases(sweep_seed):
    """dq_compress_kv over random formats (factor shapes, code widths, groups, level sets, two and
    three local tensors), call shapes (short blocks, per-sequence row counts with zeros, skipped
    sequences) and wave counts: the oracle's properties on every block where the fp32 rows are kept
    (two local tensors), and the cache written without them equal bit for bit."""
    from test_gpu_compress_direct import _both_ways
    from test_gpu_parity import _check_compress
    rng = np.random.default_rng(5000 + sweep_seed)
    for case in range(12):
        d = int(rng.choice([128, 128, 64]))
        j1 = (16 if d == 128 else 8) if rng.integers(0, 5) else int(rng.choice([8, 16] if d == 64 else [8, 32]))
        bits = int(rng.choice([2, 4, 8]))
        group = int(rng.choice([g for g in (32, 64, 128) if g <= d and (g == d or g <= d // 2) and (g * bits) % 32 == 0]))
        tb = int(rng.choice([128, 256]))
        batch, kvh = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 4, 5, 6]))
        i3, levels = int(rng.choice([1, 1, 8])), int(rng.choice([0, 1]))
        t_new = int(rng.choice([tb, tb, int(rng.integers(1, tb + 1))]))
        n_valid = None if rng.integers(0, 2) else [int(rng.choice([0, 1, 2, t_new, int(rng.integers(1, t_new + 1))]))
                                                   for _ in range(batch)]
        waves = int(rng.choice([0, 1, 2, 4]))
        w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, head_dim=d,
                                j1=j1, j2=d // j1, bits=bits, group=group, block_tokens=tb, max_seq=tb, min_seq=tb,
                                seed=7000 + 100 * sweep_seed + case, n_outlier=int(rng.choice([0, 2, 6])), i3=i3, levels=levels)
        print("compress seed %d case %d: d=%d j1=%d bits=%d G=%d Tb=%d B=%d H=%d i3=%d levels=%d t_new=%d n_valid=%s waves=%d"
              % (sweep_seed, case, d, j1, bits, group, tb, batch, kvh, i3, levels, t_new, n_valid, waves), flush=True)
        if i3 == 1 and batch <= 3:
            _check_compress(w, t_new, n_valid if n_valid is not None and all(v > 0 for v in n_valid) else None, waves=waves)
        blk = [int(rng.choice([0, 1, -1])) for _ in range(batch)]
        _both_ways(w, t_new, n_valid, blk, waves=waves)


def test_random_compress_three_tensor_cases(sweep_seed):
    """dq_compress_kv with three local tensors over random formats and call shapes, every block held
    to the oracle's properties (orthonormal columns of T_2, exact product, the oracle's quantizer on
    the GPU's own T_2 bit for bit, half-step bound): the three launches (the library's choice for a
    small call, or a forced wave count of 2 or 4) and the build that does everything in one launch
    (a forced wave count of 1; formats it does not cover fall back to the three launches)."""
    from test_gpu_mpo3 import _check_compress3
    rng = np.random.default_rng(9000 + sweep_seed)
    for case in range(8):
        d = int(rng.choice([128, 128, 128, 64]))
        j1 = 16 if d == 128 and rng.integers(0, 6) else int(rng.choice([8, 16] if d == 64 else [8, 32]))
        bits = int(rng.choice([2, 4, 8]))
        group = int(rng.choice([g for g in (32, 64, 128) if g <= d and (g == d or g <= d // 2) and (g * bits) % 32 == 0]))
        tb = int(rng.choice([128, 256]))
        batch, kvh = int(rng.choice([2, 3])), int(rng.choice([1, 2, 5]))
        levels = int(rng.choice([0, 1]))
        t_new = int(rng.choice([tb, tb, int(rng.integers(1, tb + 1))]))
        n_valid = None if rng.integers(0, 2) else [int(rng.choice([1, 2, 8, 9, t_new, int(rng.integers(1, t_new + 1))])) for _ in range(batch)]
        waves = int(rng.choice([1, 1, 0, 2, 4]))
        w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, head_dim=d,
                                j1=j1, j2=d // j1, bits=bits, group=group, block_tokens=tb, max_seq=tb, min_seq=tb, levels=levels,
                                seed=9000 + 100 * sweep_seed + case, n_outlier=int(rng.choice([0, 2, 6])), i3=8)
        print("compress3 seed %d case %d: d=%d j1=%d bits=%d G=%d Tb=%d B=%d H=%d levels=%d t_new=%d n_valid=%s waves=%d"
              % (sweep_seed, case, d, j1, bits, group, tb, batch, kvh, levels, t_new, n_valid, waves), flush=True)
        _check_compress3(w, t_new, n_valid, waves=waves)
