"""dq_attn_decode_static, the decode entry point that takes no workspace and allocates nothing: its
split partials and tickets live in a device array inside the library.  It must give the bits of
dq_attn_decode / dq_attn_decode_tail (same kernels, same launch shape) on two calls in a row, the
second one smaller, with launch shapes that do go through the scratch memory (several workgroups per
(sequence, kv head)), and refuse sizes beyond its limit without launching anything."""
import ctypes as C
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, oracle_cache_for_pairs, tolerance

pytestmark = pytest.mark.gpu


def _case(batch, kvh, rep, max_seq, lens, splits, use_tail, seed, bits=4, group=128):
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh * rep, kv_heads=kvh,
                            max_seq=max_seq, min_seq=max_seq, bits=bits, group=group, seed=seed)
    fmt, ofmt = formats(w)
    lens = np.array(lens, np.int32)
    pairs = [(b, h) for b in range(batch) for h in range(kvh)]
    cache = oracle_cache_for_pairs(w, ofmt, pairs, lens, seed=seed)
    q = workloads.query(w)
    rng = np.random.default_rng(seed)
    cap = 128
    kt = (rng.standard_normal((batch, kvh, cap, 128)) * 2).astype(np.float16)
    vt = (rng.standard_normal((batch, kvh, cap, 128)) * 2).astype(np.float16)
    tl = rng.integers(0, cap + 1, size=batch).astype(np.int32)
    if use_tail:
        want = O.attention_decode(cache, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
    else:
        want = O.attention_decode(cache, ofmt, q, lens)
    dcache = dq.cache_from_numpy(fmt, cache, DEV)
    qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
    tail = (torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV)) if use_tail else None
    ws = dq.decode_workspace(fmt, batch, w.q_heads, kvh, max_seq, DEV)
    return dict(w=w, cache=dcache, q=qd, lens=ld, tail=tail, ws=ws, want=want, max_seq=max_seq,
                flags=dq.decode_flags(splits=splits))


def _run_both(c, kernel):
    flags = c["flags"] | kernel
    print("no-alloc decode: B=%d Hq=%d Hkv=%d max_seq=%d flags=%#x tail=%s"
          % (c["w"].batch, c["w"].q_heads, c["w"].kv_heads, c["max_seq"], flags, c["tail"] is not None), flush=True)
    shape = c["q"].shape
    ref32 = torch.empty(shape, dtype=torch.float32, device=DEV)
    got32 = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    ref = dq.attn_decode(c["cache"], c["q"], c["lens"], c["max_seq"], c["ws"], out_f32=ref32, flags=flags, tail=c["tail"])
    got = dq.attn_decode(c["cache"], c["q"], c["lens"], c["max_seq"], None, out_f32=got32, flags=flags, tail=c["tail"])
    torch.cuda.synchronize()
    assert torch.equal(ref.view(torch.int16), got.view(torch.int16))
    assert torch.equal(ref32.view(torch.int32), got32.view(torch.int32))
    err = np.abs(got.cpu().numpy().astype(np.float64) - c["want"])
    assert (err <= tolerance(c["want"])).all(), err.max()


@pytest.mark.parametrize("kernel", [dq.DECODE_AUTO, dq.DECODE_FORCE_GENERIC])
def test_two_calls_in_a_row_the_second_smaller(kernel):
    big = _case(batch=3, kvh=4, rep=4, max_seq=2176, lens=[2176, 1300, 129], splits=5, use_tail=True, seed=901)
    small = _case(batch=2, kvh=2, rep=1, max_seq=640, lens=[640, 77], splits=3, use_tail=False, seed=902)
    _run_both(big, kernel)
    _run_both(small, kernel)     # the scratch memory still holds the first call's partials
    _run_both(big, kernel)       # and back again
    # the library's own launch shape (small problems are split without being told to)
    auto = _case(batch=1, kvh=2, rep=2, max_seq=4096, lens=[4000], splits=0, use_tail=True, seed=903, bits=2, group=64)
    _run_both(auto, kernel)


def test_sizes_beyond_the_limit_are_refused():
    fmt = dq.Format(4, 128, 128, 16, 8, 128)
    cache = dq.alloc_cache(fmt, 33, 16, 1, DEV)          # 33 * 16 = 528 (sequence, head) pairs > 512
    q = torch.zeros((33, 16, 128), dtype=torch.float16, device=DEV)
    lens = torch.zeros(33, dtype=torch.int32, device=DEV)
    out = torch.full_like(q, 7.0)
    with pytest.raises(dq.DQError, match="limit"):
        dq.attn_decode(cache, q, lens, 128, None, out=out)
    torch.cuda.synchronize()
    assert (out == 7.0).all()                            # nothing ran
    ok = dq.alloc_cache(fmt, 32, 16, 1, DEV)             # 512 pairs: accepted
    q2 = torch.zeros((32, 16, 128), dtype=torch.float16, device=DEV)
    out2 = dq.attn_decode(ok, q2, torch.zeros(32, dtype=torch.int32, device=DEV), 128, None)
    torch.cuda.synchronize()
    assert (out2 == 0).all()                             # empty sequences give zeros
