"""Quantization-error study on the synthetic stand-ins (Section 4.3 "Effectiveness of Tensor
Quantization"; the RTN baseline of Section 4.1): DecoQuant (quantize the large local tensor only)
against plain group round-to-nearest on the matrix itself (the same format with T_S = I), on the
value distributions of the benchmark workloads, from the oracle alone.

TEST INFRASTRUCTURE like the rest of this folder: run it as `python -m oracle.error_study` to print
the table the design notes quote; `tests/test_oracle_error_study.py` runs it and pins the directions.

Two measures per (workload distribution, code width, level set, strategy):
  * relative reconstruction error ||X - X_hat||_F / ||X||_F over `n_blocks` blocks;
  * relative error of the decode-attention output against dense fp64 attention on the original
    fp16 rows, ||out - out_dense|| / ||out_dense|| over `n_heads` (sequence, head) pairs of
    `n_tokens` tokens each.
"""
from __future__ import annotations

import dataclasses

import numpy as np

import workloads
from oracle import decoquant_oracle as O


def study(name: str, bits: int, group: int, levels: int, n_blocks: int = 12, n_heads: int = 8, n_tokens: int = 1024):
    w = dataclasses.replace(workloads.get_workload(name), bits=bits, group=group, levels=levels, max_seq=n_tokens,
                            min_seq=n_tokens, batch=2, q_heads=n_heads // 2, kv_heads=n_heads // 2)
    fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, 1, w.levels)
    tb = w.block_tokens
    out = {}
    q = workloads.query(w)
    for strategy, identity in (("decoquant", False), ("rtn", True)):
        num = den = 0.0
        blocks_done = 0
        a_num = a_den = 0.0
        for b in range(w.batch):
            for h in range(w.kv_heads):
                k, v = workloads.kv_pair(w, b, h, n_tokens)
                cache = O.empty_cache(fmt, 1, 1, n_tokens // tb)
                O.compress_sequence(cache, fmt, 0, 0, k, v, identity_small=identity)
                k_hat, v_hat = O.reconstruct_sequence(cache, fmt, 0, 0, n_tokens)
                for x, x_hat in ((k, k_hat), (v, v_hat)):
                    for blk in range(n_tokens // tb):
                        if blocks_done < n_blocks:
                            xb = x[blk * tb:(blk + 1) * tb].astype(np.float64)
                            num += np.linalg.norm(xb - x_hat[blk * tb:(blk + 1) * tb]) ** 2
                            den += np.linalg.norm(xb) ** 2
                            blocks_done += 1
                got = O.dense_attention(q[b, h], k_hat, v_hat)
                want = O.dense_attention(q[b, h], k, v)
                a_num += np.linalg.norm(got - want) ** 2
                a_den += np.linalg.norm(want) ** 2
        out[strategy] = (float(np.sqrt(num / den)), float(np.sqrt(a_num / a_den)))
    return out


CASES = [("llama7b_4bit", 4, 128), ("llama7b_2bit", 2, 64)]


def table():
    rows = []
    for name, bits, group in CASES:
        for levels in (0, 1):
            r = study(name, bits, group, levels)
            rows.append((name, bits, group, levels, r["decoquant"][0], r["rtn"][0], r["decoquant"][1], r["rtn"][1]))
    return rows


def main():
    print("distribution      bits G   levels | reconstruction rel. err: DecoQuant  RTN | attention-output rel. err: DecoQuant  RTN")
    for name, bits, group, levels, rd, rr, ad, ar in table():
        print("%-17s %-4d %-3d %-6s | %27.3f  %.3f | %29.3f  %.3f"
              % (name, bits, group, "all" if levels else "Eq. 1", rd, rr, ad, ar))


if __name__ == "__main__":
    main()
