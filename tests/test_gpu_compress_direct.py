"""dq_compress_kv_ex with DQ_COMPRESS_NO_LARGE: the decomposition kernel quantizes the large tensor
itself instead of handing it to the quantizer through the workspace.  The cache must come out bit
for bit as from dq_compress_kv (codes, steps, small tensors, status words), over code widths, step
groups, level sets, block sizes, ragged and short inputs, skipped sequences, and both wave counts
the fused kernel is launched with; calls it does not cover must fall back to the ordinary kernels."""
import dataclasses

import pytest
import torch

import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _both_ways(w, t_new, n_valid, blk):
    fmt, _ = formats(w)
    k, v = workloads.kv_tensor(w, t_new)
    kd, vd = torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV)
    nv = None if n_valid is None else torch.tensor(n_valid, dtype=torch.int32, device=DEV)
    bi = torch.tensor(blk, dtype=torch.int32, device=DEV)
    out = []
    for keep in (True, False):
        cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, 2, DEV, fill=0xA5)
        ws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV)
        ws[256:].fill_(0x5A)                       # whatever the large-tensor region held before
        dq.compress_kv(cache, kd, vd, bi, nv, ws, keep_large=keep)
        torch.cuda.synchronize()
        out.append((cache, ws[:8].clone()))
    (a, sa), (b, sb) = out
    for name in a.t:
        assert torch.equal(a.t[name], b.t[name]), name
    assert torch.equal(sa, sb)
    return a


@pytest.mark.parametrize("bits,group,levels,tb,batch,kvh", [
    (4, 128, 0, 128, 8, 8),      # 128 blocks: four waves per block
    (4, 128, 0, 128, 8, 32),     # 512 blocks: two waves per block (the benchmark's call)
    (2, 64, 0, 128, 5, 8),
    (2, 64, 1, 256, 3, 4),
    (8, 128, 0, 128, 4, 40),     # 320 blocks
    (2, 64, 0, 128, 16, 32),     # 1024 blocks: one wave per block
    (4, 64, 1, 128, 2, 6),
    (8, 64, 0, 256, 2, 2),
    (2, 128, 1, 128, 3, 3),
    # heads of 64 channels, two per workgroup (group = 64 = a head's row)
    (4, -64, 0, 128, 16, 32),    # 1024 blocks = 512 pairs
    (2, -64, 1, 256, 3, 6),
    (8, -64, 0, 128, 5, 2),
])
def test_fused_quantizer_writes_the_same_cache(bits, group, levels, tb, batch, kvh):
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, bits=bits,
                            group=abs(group), levels=levels, block_tokens=tb, max_seq=tb, min_seq=tb)
    if group < 0:
        w = dataclasses.replace(w, head_dim=64, j1=8, j2=8, n_outlier=2)
    _say("fused quantizer: bits=%d G=%d levels=%d Tb=%d B=%d H=%d" % (bits, group, levels, tb, batch, kvh))
    _both_ways(w, tb, None, [1] * batch)
    n_valid = [[tb, 37, 1, 0, tb - 1, 5, 2, tb][b % 8] for b in range(batch)]
    blk = [[0, 1, 0, 1, -1, 0, 1, 0][b % 8] for b in range(batch)]
    cache = _both_ways(w, tb - 3, n_valid, blk)
    # skipped sequences and the other slot keep the fill pattern
    for b in range(batch):
        untouched = [0, 1] if (blk[b] < 0 or n_valid[b] == 0) else [1 - blk[b]]
        for s in untouched:
            assert (cache.t["k_codes"][b, :, s] == 0xA5).all(), (b, s)


def test_calls_the_fused_kernel_does_not_cover_fall_back():
    """More than 1024 blocks, three local tensors, 64-channel heads that do not pair up, groups of 32: the flag is a
    permission, not a demand; the call gives the same cache as without it."""
    base = workloads.get_workload("llama7b_4bit")
    for kw in (dict(batch=17, q_heads=32, kv_heads=32),                                   # 1088 blocks
               dict(batch=2, q_heads=4, kv_heads=4, i3=8),
               dict(batch=2, q_heads=3, kv_heads=3, head_dim=64, j1=8, j2=8, group=64),   # an odd head is left over
               dict(batch=2, q_heads=4, kv_heads=4, group=32)):
        w = dataclasses.replace(base, max_seq=128, min_seq=128, **kw)
        _say("fused quantizer, fall-back: %s" % kw)
        _both_ways(w, 128, None, [0] * w.batch)
