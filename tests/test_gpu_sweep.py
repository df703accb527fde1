"""Seeded random sweep of the decode entry points against the oracle: code widths, group sizes,
head groupings, block sizes, ragged lengths (0, 1, around a tile edge, full), fp16 tails of every
length and capacity, and forced launch shapes (splits per sequence, waves per workgroup), so that
every tail mode and merge path of the matrix-core kernel and the plain kernel is exercised."""
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
