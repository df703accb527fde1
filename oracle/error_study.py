"""Quantization-error study on the synthetic stand-ins (Section 4.3 "Effectiveness of Tensor
Quantization"; the RTN baseline of Section 4.1): DecoQuant (quantize the large local tensor only)
against plain group round-to-nearest on the matrix itself (the same format with T_S = I), on the
value distributions of the benchmark workloads, from the oracle alone.

TEST INFRASTRUCTURE like the rest of this folder: run it as `python -m oracle.error_study` to print
the table the design notes quote; `tests/test_oracle_error_study.py` runs it and pins the directions.

A second table follows Section 4.3 "Analysis of Length of Local Tensors": the same two measures for
two, three and four local tensors (factor shapes I = 1 * T_b, 1 * (T_b/8) * 8, 1 * (T_b/16) * 4 * 4),
on the workload's rows as drawn (independent tokens) and on the same rows made to resemble their
neighbours (first-order autoregression along the tokens, coefficient 0.95), which is where a tensor
on the token side has something to absorb.

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


def _smooth_along_tokens(x: np.ndarray, rho: float) -> np.ndarray:
    """x_t <- rho * x_(t-1) + sqrt(1 - rho^2) * x_t down the rows (same variance, neighbours alike)."""
    y = np.asarray(x, dtype=np.float64).copy()
    for t in range(1, y.shape[0]):
        y[t] = rho * y[t - 1] + np.sqrt(1.0 - rho * rho) * y[t]
    return y.astype(np.float16)


def study(name: str, bits: int, group: int, levels: int, n_blocks: int = 12, n_heads: int = 8, n_tokens: int = 1024,
          strategies=None, rho: float = 0.0):
    """strategies: (label, i3, i4, identity small tensor) per row of the result; default DecoQuant
    with two local tensors against plain RTN.  rho > 0: rows smoothed along the tokens first."""
    w = dataclasses.replace(workloads.get_workload(name), bits=bits, group=group, levels=levels, max_seq=n_tokens,
                            min_seq=n_tokens, batch=2, q_heads=n_heads // 2, kv_heads=n_heads // 2)
    tb = w.block_tokens
    out = {}
    q = workloads.query(w)
    for strategy, i3, i4, identity in (strategies or (("decoquant", 1, 1, False), ("rtn", 1, 1, True))):
        fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens, i3, w.levels, 1, i4)
        num = den = 0.0
        blocks_done = 0
        a_num = a_den = 0.0
        for b in range(w.batch):
            for h in range(w.kv_heads):
                k, v = workloads.kv_pair(w, b, h, n_tokens)
                if rho > 0.0:
                    k, v = _smooth_along_tokens(k, rho), _smooth_along_tokens(v, rho)
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


LENGTHS = (("n=2", 1, 1, False), ("n=3", 8, 1, False), ("n=4", 4, 4, False), ("rtn", 1, 1, True))


def length_table(n_heads: int = 8, n_tokens: int = 1024):
    """Rows (distribution, bits, G, rho, {label: (reconstruction, attention)}) for two, three and four
    local tensors and plain RTN."""
    rows = []
    for name, bits, group in CASES:
        for rho in (0.0, 0.95):
            rows.append((name, bits, group, rho, study(name, bits, group, 0, n_heads=n_heads, n_tokens=n_tokens,
                                                        strategies=LENGTHS, rho=rho)))
    return rows


def main():
    print("distribution      bits G   levels | reconstruction rel. err: DecoQuant  RTN | attention-output rel. err: DecoQuant  RTN")
    for name, bits, group, levels, rd, rr, ad, ar in table():
        print("%-17s %-4d %-3d %-6s | %27.3f  %.3f | %29.3f  %.3f"
              % (name, bits, group, "all" if levels else "Eq. 1", rd, rr, ad, ar))
    print()
    print("distribution      bits G   tokens      | reconstruction rel. err: n=2    n=3    n=4    RTN | attention-output rel. err: n=2    n=3    n=4    RTN")
    for name, bits, group, rho, r in length_table():
        print("%-17s %-4d %-3d %-11s | %29.3f  %.3f  %.3f  %.3f | %31.3f  %.3f  %.3f  %.3f"
              % (name, bits, group, "as drawn" if rho == 0.0 else "AR(1) %.2f" % rho,
                 r["n=2"][0], r["n=3"][0], r["n=4"][0], r["rtn"][0], r["n=2"][1], r["n=3"][1], r["n=4"][1], r["rtn"][1]))


if __name__ == "__main__":
    main()
