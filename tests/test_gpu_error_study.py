"""The attention-error comparison of the quantization study (Section 4.3; RTN baseline of Section 4.1)
through the HIP path: the same rows stored as DecoQuant blocks (compressed by the GPU) and as plain
group round-to-nearest blocks (T_S = I, written by the oracle), decoded by the GPU kernels, against
dense fp64 attention on the original rows.  The GPU must report the oracle's own figures."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import decoquant_oracle as O
from oracle import error_study
import paper_2405_12591_amd as dq
import workloads
from gpu_util import DEV, formats

pytestmark = pytest.mark.gpu


def test_attention_error_decoquant_against_plain_rtn_through_the_hip_path():
    n_tok, heads = 1024, 8
    w = dataclasses.replace(workloads.get_workload("llama7b_4bit"), max_seq=n_tok, min_seq=n_tok, batch=2,
                            q_heads=heads // 2, kv_heads=heads // 2)
    fmt, ofmt = formats(w)
    k, v = workloads.kv_tensor(w)
    q = workloads.query(w)
    lens = np.full(2, n_tok, np.int32)
    dense = np.stack([np.stack([O.dense_attention(q[b, h], k[b, h], v[b, h]) for h in range(w.kv_heads)]) for b in range(2)])
    qd, ld = torch.from_numpy(q).to(DEV), torch.from_numpy(lens).to(DEV)
    ws = dq.decode_workspace(fmt, 2, w.q_heads, w.kv_heads, n_tok, DEV)
    # DecoQuant: compressed by the GPU
    cache = dq.alloc_cache(fmt, 2, w.kv_heads, n_tok // 128, DEV)
    cws = dq.compress_workspace(fmt, 2, w.kv_heads, DEV, t_new=n_tok)
    dq.compress_kv_blocks(cache, torch.from_numpy(k).to(DEV), torch.from_numpy(v).to(DEV),
                          torch.zeros(2, dtype=torch.int32, device=DEV), None, cws)
    # plain round-to-nearest: the same format with T_S = I, written by the oracle
    rtn = O.empty_cache(ofmt, 2, w.kv_heads, n_tok // 128)
    for b in range(2):
        for h in range(w.kv_heads):
            O.compress_sequence(rtn, ofmt, b, h, k[b, h], v[b, h], identity_small=True)
    rtn_d = dq.cache_from_numpy(fmt, rtn, DEV)
    rel = {}
    for name, c in (("decoquant", cache), ("rtn", rtn_d)):
        for flags in (dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC):
            o32 = torch.empty((2, w.q_heads, 128), dtype=torch.float32, device=DEV)
            dq.attn_decode(c, qd, ld, n_tok, ws, out_f32=o32, flags=flags)
            torch.cuda.synchronize()
            got = o32.cpu().numpy().astype(np.float64)
            rel[name, flags] = float(np.linalg.norm(got - dense) / np.linalg.norm(dense))
    want = error_study.study("llama7b_4bit", 4, 128, 0)
    print("attention-output error vs dense attention, 8 heads x 1024 tokens, 4-bit G128: GPU DecoQuant %.4f (oracle %.4f), "
          "GPU plain RTN %.4f (oracle %.4f)" % (rel["decoquant", 2], want["decoquant"][1], rel["rtn", 2], want["rtn"][1]), flush=True)
    for flags in (dq.DECODE_FORCE_MFMA, dq.DECODE_FORCE_GENERIC):
        # plain RTN: the GPU reads the oracle's own cache, the figures agree to the kernels' rounding
        assert abs(rel["rtn", flags] - want["rtn"][1]) <= 1e-3 * want["rtn"][1]
        # DecoQuant: the GPU's decomposition is its own (signs, rounding), the error is the same size
        assert abs(rel["decoquant", flags] - want["decoquant"][1]) <= 0.1 * want["decoquant"][1]
        assert rel["decoquant", flags] < rel["rtn", flags]
