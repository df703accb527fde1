"""Synthetic stand-ins for LLaMA-family KV caches.

The paper evaluates on LLaMA / OPT key and value activations, which are not
available offline; these generators reproduce the structure that matters for
the method (Section 3.1: a few outlier channels with a much wider range than
the bulk) with seeded random numbers.

Every (sequence b, kv head h) pair owns an independent PCG64 stream derived
from (seed, tag, b, h), so a test can draw a few pairs without generating the
whole layer, and the GPU harness, which draws all of them, gets the same bits.
Values are drawn in fp32, clipped to |x| <= 512 and rounded to fp16.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

CLIP = 512.0
_TAG_KV, _TAG_Q, _TAG_LEN, _TAG_CH, _TAG_NEW = 11, 12, 13, 14, 15


@dataclass(frozen=True)
class Workload:
    """Shape, value distribution and storage format of one configuration."""
    name: str
    seed: int
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    max_seq: int            # tokens per sequence (upper bound when lengths are mixed)
    min_seq: int            # == max_seq unless lengths are mixed
    bits: int
    group: int
    j1: int
    j2: int
    block_tokens: int
    dist: str               # "normal" | "lognormal_tokens" | "layer_outliers" | "student_t"
    n_outlier: int          # outlier channels per head (or per layer for layer_outliers)
    outlier_scale: float
    append_tokens: int = 0  # tokens appended (and compressed) before the decode step
    i3: int = 1             # 8: three local tensors (the third one 8 x 8 on the token side)
    levels: int = 0         # 1: the quantizer's non-default level set (all 2^bits codes)
    i1: int = 1             # 2 or 4: a token factor on the small tensor (Eq. 2 with i_1 > 1)


WORKLOADS = {
    "tiny": Workload("tiny", 1001, 1, 4, 4, 64, 256, 256, 4, 64, 8, 8, 256,
                     "normal", 2, 20.0),
    "llama7b_4bit": Workload("llama7b_4bit", 1002, 8, 32, 32, 128, 4096, 4096, 4, 128, 16, 8, 128,
                             "lognormal_tokens", 4, 20.0),
    "llama7b_2bit": Workload("llama7b_2bit", 1003, 16, 32, 32, 128, 8192, 8192, 2, 64, 16, 8, 128,
                             "lognormal_tokens", 4, 20.0),
    "llama13b_mixed": Workload("llama13b_mixed", 1004, 4, 40, 40, 128, 16384, 8192, 4, 128, 16, 8, 128,
                               "layer_outliers", 51, 30.0, append_tokens=128),
    "gqa_long": Workload("gqa_long", 1005, 16, 32, 8, 128, 32768, 32768, 4, 128, 16, 8, 128,
                         "student_t", 4, 10.0),
    # the 8-bit variant of the benchmark shape (the paper's fused kernel covers 2, 4 and 8 bits)
    "llama7b_8bit": Workload("llama7b_8bit", 1006, 8, 32, 32, 128, 4096, 4096, 8, 128, 16, 8, 128,
                             "lognormal_tokens", 4, 20.0),
    # eight query heads per kv head (the head grouping of the 70B-class LLaMA models) on the long-context shape
    "gqa8_long": Workload("gqa8_long", 1008, 16, 64, 8, 128, 32768, 32768, 4, 128, 16, 8, 128,
                          "student_t", 4, 10.0),
    # heads of 64 channels (the head size of the smaller OPT models the paper evaluates): same cached
    # tokens per sequence and about the same bytes per launch as the benchmark shape
    "opt_d64_4bit": Workload("opt_d64_4bit", 1009, 16, 32, 32, 64, 4096, 4096, 4, 64, 8, 8, 128,
                             "lognormal_tokens", 2, 20.0),
    # the benchmark shape with three local tensors (the paper's n = 3 variant)
    "llama7b_4bit_n3": Workload("llama7b_4bit_n3", 1007, 8, 32, 32, 128, 4096, 4096, 4, 128, 16, 8, 128,
                                "lognormal_tokens", 4, 20.0, i3=8),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *key])))


def _outlier_channels(w: Workload, which: int, h: int) -> np.ndarray:
    """Outlier channel indices of kv head h (fixed over tokens and batch).

    which: 0 for keys, 1 for values (each tensor has its own outlier channels).
    """
    if w.dist == "layer_outliers":
        # a fixed number of (head, channel) pairs drawn without replacement over the layer
        r = _rng(w.seed, _TAG_CH, which)
        flat = r.choice(w.kv_heads * w.head_dim, size=w.n_outlier, replace=False)
        return np.sort(flat[flat // w.head_dim == h] % w.head_dim)
    r = _rng(w.seed, _TAG_CH, which, h)
    return np.sort(r.choice(w.head_dim, size=w.n_outlier, replace=False))


def _draw(w: Workload, r: np.random.Generator, n_tok: int, ch: np.ndarray) -> np.ndarray:
    x = r.standard_normal((n_tok, w.head_dim), dtype=np.float32)
    if w.dist == "lognormal_tokens":
        x *= np.exp(0.5 * r.standard_normal((n_tok, 1), dtype=np.float32))
    if w.dist == "student_t":
        if ch.size:
            x[:, ch] += np.float32(w.outlier_scale) * r.standard_t(3.0, size=(n_tok, ch.size)).astype(np.float32)
    else:
        x[:, ch] *= np.float32(w.outlier_scale)
    np.clip(x, -CLIP, CLIP, out=x)
    return x.astype(np.float16)


def kv_pair(w: Workload, b: int, h: int, n_tok: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """fp16 K and V of shape [n_tok, head_dim] for sequence b, kv head h."""
    n = w.max_seq if n_tok is None else n_tok
    r = _rng(w.seed, _TAG_KV, b, h)
    k = _draw(w, r, w.max_seq, _outlier_channels(w, 0, h))
    v = _draw(w, r, w.max_seq, _outlier_channels(w, 1, h))
    return k[:n], v[:n]


def appended_pair(w: Workload, b: int, h: int) -> Tuple[np.ndarray, np.ndarray]:
    """fp16 K and V rows [append_tokens, head_dim] appended after the cached tokens."""
    r = _rng(w.seed, _TAG_NEW, b, h)
    k = _draw(w, r, w.append_tokens, _outlier_channels(w, 0, h))
    v = _draw(w, r, w.append_tokens, _outlier_channels(w, 1, h))
    return k, v


def kv_tensor(w: Workload, n_tok: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Whole layer: fp16 K, V of shape [batch, kv_heads, n_tok, head_dim]."""
    n = w.max_seq if n_tok is None else n_tok
    k = np.empty((w.batch, w.kv_heads, n, w.head_dim), np.float16)
    v = np.empty_like(k)
    for b in range(w.batch):
        for h in range(w.kv_heads):
            k[b, h], v[b, h] = kv_pair(w, b, h, n)
    return k, v


def query(w: Workload) -> np.ndarray:
    """One fp16 decode query per (sequence, query head): [batch, q_heads, head_dim]."""
    r = _rng(w.seed, _TAG_Q)
    return r.standard_normal((w.batch, w.q_heads, w.head_dim), dtype=np.float32).astype(np.float16)


def seq_lens(w: Workload) -> np.ndarray:
    """int32 [batch] cached tokens per sequence (uniform integers in [min_seq, max_seq])."""
    if w.min_seq == w.max_seq:
        return np.full(w.batch, w.max_seq, np.int32)
    r = _rng(w.seed, _TAG_LEN)
    return r.integers(w.min_seq, w.max_seq + 1, size=w.batch).astype(np.int32)
