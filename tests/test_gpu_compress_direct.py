"""dq_compress_kv_ex with DQ_COMPRESS_NO_LARGE: the decomposition kernel quantizes the large tensor
itself instead of handing it to the quantizer through the workspace.  The cache must come out bit
for bit as from dq_compress_kv (codes, steps, small tensors, status words), over code widths, step
groups, level sets, block sizes, ragged and short inputs, skipped sequences, and both wave counts
the fused kernel is launched with; calls it does not cover must fall back to the ordinary kernels."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _both_ways(w, t_new, n_valid, blk, waves=0):
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
        dq.compress_kv(cache, kd, vd, bi, nv, ws, keep_large=keep, waves=waves)
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


@pytest.mark.parametrize("name,batch,kvh", [("llama13b_mixed", 4, 40), ("llama7b_4bit", 8, 32), ("llama7b_2bit", 16, 32)])
def test_properties_at_the_call_sizes_that_ship(name, batch, kvh):
    """Calls of 320, 512 and 1024 blocks (the 13B-shaped configuration's appended rows, the benchmark's
    companion step, the 2-bit configuration's) with the library's own choice of waves per block: on
    sampled blocks the two-kernel path's output has the properties the paper fixes (orthonormal rows
    of T_L, exact factorisation, codes and steps equal to the oracle's quantization of the GPU's own
    T_L, reconstruction within the half-step bound); the one-kernel path then writes the same cache
    bit for bit, so the same holds for it."""
    from oracle import decoquant_oracle as O
    from test_gpu_parity import block_properties
    w = dataclasses.replace(workloads.get_workload(name), batch=batch, q_heads=kvh, kv_heads=kvh, max_seq=128, min_seq=128,
                            append_tokens=0)
    fmt, ofmt = formats(w)
    _say("compress properties at %d blocks per call (%s)" % (2 * batch * kvh, name))
    gen = torch.Generator(device=DEV).manual_seed(11)
    kd = (torch.randn((batch, kvh, 128, 128), device=DEV, generator=gen) * 1.5).to(torch.float16)
    vd = (torch.randn((batch, kvh, 128, 128), device=DEV, generator=gen) * 1.5).to(torch.float16)
    sample = [(0, 0), (batch - 1, kvh - 1), (1, 5), (batch // 2, kvh // 2), (2, kvh - 2), (batch - 1, 0)]
    host = {}
    for b, h in sample:                                  # the workload's rows (outlier channels and all)
        kk, vv = workloads.kv_pair(w, b, h, 128)
        host[b, h] = (kk, vv)
        kd[b, h], vd[b, h] = torch.from_numpy(kk).to(DEV), torch.from_numpy(vv).to(DEV)
    n_valid = torch.full((batch,), 128, dtype=torch.int32, device=DEV)
    n_valid[1] = 77                                      # one ragged sequence
    slot = torch.zeros(batch, dtype=torch.int32, device=DEV)
    caches = []
    for keep in (True, False):
        cache = dq.alloc_cache(fmt, batch, kvh, 1, DEV, fill=0xA5)
        ws = dq.compress_workspace(fmt, batch, kvh, DEV)
        dq.compress_kv(cache, kd, vd, slot, n_valid, ws, keep_large=keep)
        torch.cuda.synchronize()
        assert int(ws[:4].view(torch.int32).item()) == 0
        caches.append((cache, ws))
    (two, ws2), (one, _) = caches
    for n in two.t:
        assert torch.equal(two.t[n], one.t[n]), n
    arrs = {n: t.cpu().numpy() for n, t in two.t.items()}
    units = batch * kvh * 2
    large = ws2[256:256 + 4 * units * 128 * 128].view(torch.float32).cpu().numpy().reshape(units, 128, 128)
    worst = 0.0
    for b, h in sample:
        for which, rows in (("k", host[b, h][0]), ("v", host[b, h][1])):
            nv = 77 if b == 1 else 128
            x = np.zeros((128, 128))
            x[:nv] = rows[:nv].astype(np.float64)
            worst = max(worst, block_properties(arrs, ofmt, x, large[(b * kvh + h) * 2 + (which == "v")], b, h, 0, which))
    _say("  worst |T_L T_L^T - I| = %.3g over %d sampled blocks" % (worst, 2 * len(sample)))


@pytest.mark.parametrize("bits,group,levels,d", [(4, 128, 0, 128), (2, 64, 1, 128), (8, 128, 0, 128), (4, 64, 0, 64)])
def test_the_lean_build_for_large_calls_writes_the_same_bits(bits, group, levels, d):
    """Calls of more than 1024 blocks take a build of the decomposition kernel that keeps fewer
    registers and less LDS (several blocks per SIMD).  Same arithmetic: with and without the fp32
    rows kept, the cache must equal, bit for bit, what the one-wave build of the small calls writes
    (selected through the flags word), ragged rows and skipped sequences included."""
    batch, kvh = 9, 64 if d == 64 else 32
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), batch=batch, q_heads=kvh, kv_heads=kvh, bits=bits,
                            group=group, levels=levels, max_seq=256, min_seq=256, head_dim=d, j1=d // 8, j2=8)
    fmt, _ = formats(w)
    units = batch * kvh * 2 * 2
    _say("lean build: bits=%d G=%d levels=%d d=%d, %d blocks per call" % (bits, group, levels, d, units))
    gen = torch.Generator(device=DEV).manual_seed(3)
    kd = (torch.randn((batch, kvh, 256, d), device=DEV, generator=gen) * 2).to(torch.float16)
    vd = (torch.randn((batch, kvh, 256, d), device=DEV, generator=gen) * 2).to(torch.float16)
    kd[:, :, :, 5] *= 20
    n_valid = torch.tensor([256, 130, 1, 0, 255, 128, 129, 256, 77][:batch], dtype=torch.int32, device=DEV)
    first = torch.tensor([0, 1, 0, 0, 0, -1, 0, 0, 1][:batch], dtype=torch.int32, device=DEV)
    out = []
    for keep, waves in ((True, 0), (False, 0), (True, 1), (False, 1)):
        cache = dq.alloc_cache(fmt, batch, kvh, 2, DEV, fill=0xA5)
        ws = dq.compress_workspace(fmt, batch, kvh, DEV, t_new=256)
        dq.compress_kv_blocks(cache, kd, vd, first, n_valid, ws, keep_large=keep, waves=waves)
        torch.cuda.synchronize()
        out.append((cache, ws[:8].clone()))
    for cache, status in out[1:]:
        for name in cache.t:
            assert torch.equal(cache.t[name], out[0][0].t[name]), name
        assert torch.equal(status, out[0][1])
