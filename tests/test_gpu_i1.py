"""Factor shapes with a token factor on the small tensor (format.i1 = 2 or 4; Preliminary, Eq. 2 with
n = 2 and i_1 > 1) through the C ABI: compression checked through the oracle's properties, decode
against the oracle on oracle-compressed and on GPU-compressed caches, ragged lengths, fp16 tails and
forced sequence splits."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats, oracle_cache_for_pairs, tolerance, run_decode
from test_gpu_parity import _check_compress, _decode_case

pytestmark = pytest.mark.gpu

SHAPES = [  # (i1, j1, d, bits, group, T_b)
    (2, 16, 128, 4, 128, 128),
    (2, 8, 128, 2, 64, 256),
    (4, 8, 128, 8, 128, 128),
    (2, 8, 64, 4, 64, 128),
    (4, 8, 64, 4, 32, 256),
    (2, 16, 64, 2, 64, 128),
]


def _w(i1, j1, d, bits, group, tb, **kw):
    base = dict(head_dim=d, j1=j1, j2=d // j1, bits=bits, group=group, block_tokens=tb, i1=i1,
                n_outlier=2 if d == 64 else 4)
    base.update(kw)
    return dataclasses.replace(workloads.get_workload("llama7b_4bit"), **base)


@pytest.mark.parametrize("shape", SHAPES)
def test_the_matrix_core_kernel_declines_and_the_plain_one_decodes(shape):
    w = _w(*shape, batch=3, q_heads=4, kv_heads=2, max_seq=3 * shape[5], min_seq=3 * shape[5], seed=7100 + shape[0])
    fmt, _ = formats(w)
    assert not dq.decode_mfma_supported(fmt, w.q_heads, w.kv_heads)
    tb = shape[5]
    lens = [3 * tb, 0, tb + 1]
    print("decode i1=%d j1=%d d=%d bits=%d G=%d Tb=%d lens=%s" % (*shape, lens), flush=True)
    worst = _decode_case(w, lens, dq.DECODE_AUTO)
    print("  worst fp32 abs err %.3g" % worst, flush=True)
    _decode_case(w, [1, 2 * tb - 1, tb // 2], dq.decode_flags(splits=3))


@pytest.mark.parametrize("shape", SHAPES)
def test_compress_properties(shape):
    tb = shape[5]
    w = _w(*shape, batch=3, q_heads=2, kv_heads=2, max_seq=tb, min_seq=tb, seed=7200 + shape[0])
    print("compress i1=%d j1=%d d=%d bits=%d G=%d Tb=%d" % shape, flush=True)
    _check_compress(w, tb, None)
    _check_compress(w, tb - 3, [tb - 3, 37, 1])


@pytest.mark.parametrize("shape", [SHAPES[0], SHAPES[4]])
def test_gpu_compressed_cache_with_tail_decodes_like_its_oracle_reading(shape):
    """Compress three blocks per head on the GPU (one call), then decode over them plus an fp16 tail on
    the GPU and with the oracle from the GPU's own arrays."""
    tb = shape[5]
    w = _w(*shape, batch=2, q_heads=4, kv_heads=2, max_seq=3 * tb, min_seq=3 * tb, seed=7300 + shape[0])
    fmt, ofmt = formats(w)
    k, v = workloads.kv_tensor(w)
    cache = dq.alloc_cache(fmt, w.batch, w.kv_heads, 3, DEV)
    ws = dq.compress_workspace(fmt, w.batch, w.kv_heads, DEV, t_new=3 * tb)
    lens = np.array([3 * tb, 2 * tb + 5], np.int32)
    dq.compress_kv_blocks(cache, torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV),
                          torch.zeros(2, dtype=torch.int32, device=DEV), torch.from_numpy(lens).to(DEV), ws)
    torch.cuda.synchronize()
    arrs = {n: t.cpu().numpy() for n, t in cache.t.items()}
    q = workloads.query(w)
    rng = np.random.default_rng(5)
    cap = 64
    kt = (rng.standard_normal((2, 2, cap, w.head_dim)) * 2).astype(np.float16)
    vt = (rng.standard_normal((2, 2, cap, w.head_dim)) * 2).astype(np.float16)
    tl = np.array([cap, 3], np.int32)
    want = O.attention_decode(arrs, ofmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
    dws = dq.decode_workspace(fmt, 2, w.q_heads, 2, 3 * tb, DEV)
    out = dq.attn_decode(cache, torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV), 3 * tb, dws,
                         tail=(torch.from_numpy(kt).to(DEV), torch.from_numpy(vt).to(DEV), torch.from_numpy(tl).to(DEV)))
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy().astype(np.float64) - want)
    assert (err <= tolerance(want)).all(), err.max()
    # the lossy cache approximates attention on the original rows
    for b in range(2):
        for hq in range(4):
            kk = np.concatenate([k[b, hq // 2, :lens[b]], kt[b, hq // 2, :tl[b]]])
            vv = np.concatenate([v[b, hq // 2, :lens[b]], vt[b, hq // 2, :tl[b]]])
            ref = O.dense_attention(q[b, hq], kk, vv)
            assert np.abs(want[b, hq] - ref).max() < 0.2 * np.abs(vv.astype(np.float64)).max()
