"""CPU oracle for decode attention over a DecoQuant-compressed KV cache.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what the
GPU library must compute, written from the paper (arXiv 2405.12591).  It is
imported by the tests, by the smoke check and by the benchmark's CPU-baseline
leg, never by the product path, and it shares no code with the HIP library.

Arithmetic is numpy fp64 throughout; the only roundings are the ones the
storage format fixes (fp32 hand-off of the large tensor, fp16 scales, fp16
small tensor, integer codes).

What follows which passage of the paper
  * quantizer                      Preliminary, Eq. 1 (symmetric round-to-nearest, step
                                   Delta = max|W| / (2^(m-1) - 1))
  * MPO decomposition              Preliminary, Eq. 2 (product of local tensors
                                   T_(k)[d_{k-1}, i_k, j_k, d_k], prod i_k = I, prod j_k = J)
  * n = 2 split T_L x T_S          Section 3.1, Eq. 3
  * quantize T_L only, T_S 16-bit  Section 3.1, "Local Tensor Quantization"
  * dequantize, then attention     Section 3.2 (cache recovered to floating point, then
                                   ordinary attention); "Kernel Fusion for Dequantization"
                                   (scale x integer, then the product of T_L and T_S)
  * compression ratio mu           Section 3.3, Eq. 4
  * n = 3 and n = 4 variants (T_1 x T_2 x T_3 [x T_4], T_2 quantized)
                                   Preliminary, Eq. 2 with n = 3, 4; Section 4.3 "Analysis of
                                   Length of Local Tensors"

Readings taken where the paper is silent (each is listed in the design notes of
the repository): per-head blocks of `block_tokens` rows; i_1 = 1 by default so the small
tensor mixes only channels (`i1` > 1: Eq. 2 as printed with a token factor on the small tensor,
which then is (i1*j1) x (i1*j1) and mixes i1 token groups too; the large tensor keeps the block's
row count and row length, row a2*i1 + rho holding bond slice rho of position a2); no bond truncation; singular values kept in the
small tensor; per-group fp16 steps with groups of `group` consecutive elements
inside one token row of the large tensor; ties round to even; 2-bit uses the
literal Eq. 1 levels {-1, 0, +1}; codes stored offset-binary.  Non-default level set
(`levels` = 1, not the paper's: Eq. 1 is symmetric): all 2^m codes, c in
[-2^(m-1), 2^(m-1) - 1] ({-2, -1, 0, +1} at 2 bits), with the step sized so that neither end
clips, Delta = fp16(max(max(x) / (2^(m-1) - 1), max(-x) / 2^(m-1))).  Three local tensors
(`i3` > 1): factors I = 1 * (T_b/i3) * i3, J = j1 * j2 * 1, so the third tensor mixes
the i3 tokens of a run of consecutive tokens; the singular values of the first cut stay in
T_1 and those of the second cut in T_3, which leaves the quantized middle tensor T_2 with
orthonormal columns.  Four local tensors (`i4` > 1, this module only: the HIP library has no
such format): I = 1 * i2 * i3 * i4, J = j1 * j2 * 1 * 1, three cuts, the singular values of the
second cut pushed on into the third and those of the third kept in T_4, so that the quantized T_2
again has orthonormal columns; T_3 [i3*i4, i3, i4] and T_4 [i4, i4] are kept in fp16.

Parity pins (tests/test_oracle_*.py): exact reconstruction <= 1e-10, orthonormal
rows of T_L, textbook SVD special cases, exact-rational brute force of the
quantizer, |x - Delta*c| <= Delta/2, hand-packed byte fixtures, Eq. 4 closed
form, attention == brute-force dense attention when quantization is disabled,
identity small tensor == plain group RTN, softmax invariants.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

TILE_TOKENS = 128  # value codes are stored token-contiguous inside tiles of this many tokens


@dataclass(frozen=True)
class Format:
    """Storage format of a compressed cache (mirrors the fields the C header documents)."""
    bits: int
    group: int
    head_dim: int
    j1: int
    j2: int
    block_tokens: int
    i3: int = 1   # 1: two local tensors; > 1: three, the third one i3 x i3 on the token side
    levels: int = 0   # 0: Eq. 1's symmetric codes [-qmax, qmax]; 1: all 2^bits codes [-qmax - 1, qmax]
    i1: int = 1   # Eq. 2's i_1: the small tensor's share of the token index (i_2 = block_tokens / i1);
                  # > 1: T_S is (i1*j1) x (i1*j1) and mixes i1 groups of tokens as well as channels
    i4: int = 1   # > 1 (with i3 > 1): four local tensors, the token index split as (a2, a3, a4) with
                  # a4 < i4 fastest; not a format of the HIP library

    @property
    def small_side(self) -> int:
        """Rows (= columns = bond dimension) of the small tensor: i1 * j1."""
        return self.i1 * self.j1

    def check(self) -> None:
        if self.bits not in (2, 4, 8):
            raise ValueError("bits must be 2, 4 or 8")
        if self.j1 * self.j2 != self.head_dim:
            raise ValueError("head_dim must equal j1*j2")
        if self.head_dim % self.group:
            raise ValueError("group must divide head_dim")
        if self.block_tokens % TILE_TOKENS:
            raise ValueError("block_tokens must be a multiple of %d" % TILE_TOKENS)
        if self.i3 < 1 or self.block_tokens % self.i3:
            raise ValueError("i3 must divide block_tokens")
        if self.levels not in (0, 1):
            raise ValueError("levels must be 0 (symmetric) or 1 (all codes)")
        if self.i1 < 1 or self.block_tokens % self.i1:
            raise ValueError("i1 must divide block_tokens")
        if self.i1 > 1 and self.i3 > 1:
            raise ValueError("i1 > 1 is defined for two local tensors only")
        if self.i4 < 1 or (self.i4 > 1 and (self.i3 == 1 or self.block_tokens % (self.i3 * self.i4))):
            raise ValueError("i4 > 1 needs i3 > 1 and i3*i4 dividing block_tokens")
        if self.i1 * self.j1 > (self.block_tokens // self.i1) * self.j2:
            raise ValueError("the small tensor's side must not exceed the large tensor's (bond = i1*j1)")

    @property
    def bond3(self) -> int:
        """Bond dimension between T_2 and T_3 (rows of the large tensor per position a2)."""
        return self.i3 * self.i4

    @property
    def qmax(self) -> int:
        return (1 << (self.bits - 1)) - 1

    @property
    def full_range(self) -> bool:
        return self.levels == 1

    @property
    def row_bytes(self) -> int:
        return self.head_dim * self.bits // 8

    @property
    def groups_per_row(self) -> int:
        return self.head_dim // self.group


# --------------------------------------------------------------------------------------
# Eq. 2 / Eq. 3: matricisation and the MPO decomposition
# --------------------------------------------------------------------------------------

def matricise(x: np.ndarray, i1: int, j1: int) -> np.ndarray:
    """Regroup X[I, J] as M[(a1, b1), (a2, b2)] = X[a1*i2 + a2, b1*j2 + b2]  (Eq. 2, n = 2).

    Row index of M pairs the first factor of the row index of X with the first
    factor of its column index; that pairing is what lets a two-site MPO be
    found by one SVD.
    """
    big_i, big_j = x.shape
    i2, j2 = big_i // i1, big_j // j1
    if i1 * i2 != big_i or j1 * j2 != big_j:
        raise ValueError("factor sizes must divide the matrix shape")
    return x.reshape(i1, i2, j1, j2).transpose(0, 2, 1, 3).reshape(i1 * j1, i2 * j2)


def unmatricise(m: np.ndarray, big_i: int, big_j: int, i1: int, j1: int) -> np.ndarray:
    """Inverse of `matricise`."""
    i2, j2 = big_i // i1, big_j // j1
    return m.reshape(i1, j1, i2, j2).transpose(0, 2, 1, 3).reshape(big_i, big_j)


def mpo_split(x: np.ndarray, j1: int, i1: int = 1, sigma_in: str = "small"
              ) -> Tuple[np.ndarray, np.ndarray]:
    """Two-site MPO of X (Eq. 3): returns (T_S, T_L) with matricise(X) = T_S @ T_L exactly.

    T_S is (i1*j1) x d and T_L is d x (i2*j2) with bond dimension d = min of the
    two sides (no truncation).  `sigma_in` says which factor keeps the singular
    values; "small" leaves T_L with orthonormal rows.  Each (column of T_S, row of
    T_L) pair is sign-flipped so that the largest-magnitude entry of the T_L row is
    positive; this only makes the output reproducible.
    """
    m = matricise(np.asarray(x, dtype=np.float64), i1, j1)
    u, s, vt = np.linalg.svd(m, full_matrices=False)
    if sigma_in == "small":
        t_s, t_l = u * s[None, :], vt
    elif sigma_in == "large":
        t_s, t_l = u, s[:, None] * vt
    else:
        raise ValueError("sigma_in must be 'small' or 'large'")
    piv = np.argmax(np.abs(t_l), axis=1)
    sign = np.where(t_l[np.arange(t_l.shape[0]), piv] < 0, -1.0, 1.0)
    return t_s * sign[None, :], t_l * sign[:, None]


def mpo_decompose(w: np.ndarray, ishape: Sequence[int], jshape: Sequence[int]) -> List[np.ndarray]:
    """General n-site MPO (Eq. 2) by sequential SVDs, no truncation.

    Returns local tensors T_(k) of shape [d_{k-1}, i_k, j_k, d_k] with d_0 = d_n = 1
    whose contraction over the bond indices reproduces W.  Singular values are
    pushed to the right at every step.
    """
    n = len(ishape)
    big_i, big_j = int(np.prod(ishape)), int(np.prod(jshape))
    if w.shape != (big_i, big_j) or len(jshape) != n:
        raise ValueError("shape factors do not match the matrix")
    t = np.asarray(w, dtype=np.float64).reshape(*ishape, *jshape)
    order = [ax for k in range(n) for ax in (k, n + k)]  # (i1, j1, i2, j2, ...)
    rest = t.transpose(order)
    tensors = []
    d_prev = 1
    for k in range(n - 1):
        rest = rest.reshape(d_prev * ishape[k] * jshape[k], -1)
        u, s, vt = np.linalg.svd(rest, full_matrices=False)
        d = s.shape[0]
        tensors.append(u.reshape(d_prev, ishape[k], jshape[k], d))
        rest = s[:, None] * vt
        d_prev = d
    tensors.append(rest.reshape(d_prev, ishape[-1], jshape[-1], 1))
    return tensors


def mpo_contract(tensors: Sequence[np.ndarray]) -> np.ndarray:
    """Multiply local tensors back into the matrix W[I, J] (the product in Eq. 2)."""
    acc = tensors[0]  # [1, i, j, d]
    for t in tensors[1:]:
        # acc[a, I, J, d] x t[d, i, j, e] -> [a, I, i, J, j, e]
        acc = np.einsum("aIJd,dije->aIiJje", acc, t)
        a, big_i, i, big_j, j, e = acc.shape
        acc = acc.reshape(a, big_i * i, big_j * j, e)
    return acc[0, :, :, 0]


def as_local_tensors(t_s: np.ndarray, t_l: np.ndarray, i1: int, j1: int, i2: int, j2: int
                     ) -> List[np.ndarray]:
    """View (T_S, T_L) of `mpo_split` as the two 4-index local tensors of Eq. 2."""
    d = t_s.shape[1]
    return [t_s.reshape(1, i1, j1, d), t_l.reshape(d, i2, j2, 1)]


def mpo3_split(x: np.ndarray, j1: int, i3: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Three-site MPO of X[T_b, d] (Eq. 2 with n = 3) for the factor shapes
    I = 1 * i2 * i3, J = j1 * j2 * 1:  X[(a2, a3), (b1, b2)] = sum_{r, e} T_1[b1, r] T_2[r, a2, b2, e] T_3[e, a3].

    Two SVDs, no truncation.  The first is `mpo_split` (T_1 = U S, bond r of size j1); its right
    factor, regrouped as A[(r, a2, b2), a3], is cut again: A = U' S' V'^T, T_2 = U' (orthonormal
    columns, the large tensor), T_3 = S' V'^T (i3 x i3, bond e first).  Returns
    (T_1 [j1, j1], T_2 [j1, i2, j2, i3], T_3 [i3, i3]).  Each (column of T_2, row of T_3) pair is
    sign-flipped so that the largest-magnitude entry of the T_3 row is positive (reproducibility
    only).
    """
    x = np.asarray(x, dtype=np.float64)
    n_tok, d = x.shape
    j2, i2 = d // j1, n_tok // i3
    if i2 * i3 != n_tok:
        raise ValueError("i3 must divide the number of rows")
    t_1, right = mpo_split(x, j1)                       # right[r, (t, b2)], t = a2*i3 + a3
    a = right.reshape(j1, i2, i3, j2).transpose(0, 1, 3, 2).reshape(j1 * i2 * j2, i3)
    u, s, vt = np.linalg.svd(a, full_matrices=False)
    t_3 = s[:, None] * vt
    piv = np.argmax(np.abs(t_3), axis=1)
    sign = np.where(t_3[np.arange(t_3.shape[0]), piv] < 0, -1.0, 1.0)
    return t_1, (u * sign[None, :]).reshape(j1, i2, j2, i3), t_3 * sign[:, None]


def mpo3_contract(t_1: np.ndarray, t_2: np.ndarray, t_3: np.ndarray) -> np.ndarray:
    """X[(a2, a3), (b1, b2)] from the three local tensors of `mpo3_split`, term by term."""
    j1, i2, j2, i3 = t_2.shape
    x = np.einsum("br,racd,de->aebc", t_1, t_2, t_3)    # [a2, a3, b1, b2]
    return x.reshape(i2 * i3, j1 * j2)


def mpo4_split(x: np.ndarray, j1: int, i3: int, i4: int
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Four-site MPO of X[T_b, d] (Eq. 2 with n = 4) for the factor shapes I = 1 * i2 * i3 * i4,
    J = j1 * j2 * 1 * 1 (token index (a2, a3, a4), a4 fastest):
      X[(a2, a3, a4), (b1, b2)] = sum_{r, e, f} T_1[b1, r] T_2[r, a2, b2, e] T_3[e, a3, f] T_4[f, a4].

    Three SVDs, no truncation.  The first is `mpo_split` (T_1 = U S).  Its right factor, regrouped
    as A[(r, a2, b2), (a3, a4)], is cut into T_2 = U' (orthonormal columns, bond e of size i3*i4,
    the large tensor) and S' V'^T, which, regrouped as B[(e, a3), a4], is cut into T_3 = U''
    (bond f of size i4) and T_4 = S'' V''^T.  Returns (T_1 [j1, j1], T_2 [j1, i2, j2, i3*i4],
    T_3 [i3*i4, i3, i4], T_4 [i4, i4]).  Signs: as in `mpo3_split`, fixed by the largest entry of
    the right-hand factor's row at each of the two later cuts (reproducibility only).
    """
    x = np.asarray(x, dtype=np.float64)
    n_tok, d = x.shape
    j2, run = d // j1, i3 * i4
    i2 = n_tok // run
    if i2 * run != n_tok:
        raise ValueError("i3*i4 must divide the number of rows")
    if j1 * i2 * j2 < run:
        raise ValueError("the large tensor's side must not be smaller than i3*i4")
    t_1, right = mpo_split(x, j1)                       # right[r, (t, b2)], t = (a2, a3, a4)
    a = right.reshape(j1, i2, run, j2).transpose(0, 1, 3, 2).reshape(j1 * i2 * j2, run)
    u, s, vt = np.linalg.svd(a, full_matrices=False)
    rest = s[:, None] * vt                              # [e, (a3, a4)]
    piv = np.argmax(np.abs(rest), axis=1)
    sign = np.where(rest[np.arange(run), piv] < 0, -1.0, 1.0)
    t_2 = (u * sign[None, :]).reshape(j1, i2, j2, run)
    rest = rest * sign[:, None]
    b = rest.reshape(run * i3, i4)                      # [(e, a3), a4]
    u2, s2, vt2 = np.linalg.svd(b, full_matrices=False)
    t_4 = s2[:, None] * vt2
    piv = np.argmax(np.abs(t_4), axis=1)
    sign = np.where(t_4[np.arange(i4), piv] < 0, -1.0, 1.0)
    return t_1, t_2, (u2 * sign[None, :]).reshape(run, i3, i4), t_4 * sign[:, None]


def mpo4_contract(t_1: np.ndarray, t_2: np.ndarray, t_3: np.ndarray, t_4: np.ndarray) -> np.ndarray:
    """X[(a2, a3, a4), (b1, b2)] from the four local tensors of `mpo4_split`, term by term."""
    j1, i2, j2, run = t_2.shape
    _, i3, i4 = t_3.shape
    x = np.einsum("br,racd,def,fg->aegbc", t_1, t_2, t_3, t_4)   # [a2, a3, a4, b1, b2]
    return x.reshape(i2 * i3 * i4, j1 * j2)


def middle_to_token_major(t_2: np.ndarray) -> np.ndarray:
    """T_2[r, a2, b2, e] -> rows (a2, e), elements r*j2 + b2, rounded to fp32: the same row layout
    as the two-tensor large tensor, with the bond index e in the place of the token a3."""
    j1, i2, j2, i3 = t_2.shape
    return np.ascontiguousarray(t_2.transpose(1, 3, 0, 2).reshape(i2 * i3, j1 * j2)).astype(np.float32)


def token_major_to_middle(kp: np.ndarray, j1: int, j2: int, i3: int) -> np.ndarray:
    """Inverse layout change of `middle_to_token_major` (values untouched)."""
    i2 = kp.shape[0] // i3
    return kp.reshape(i2, i3, j1, j2).transpose(2, 0, 3, 1)


# --------------------------------------------------------------------------------------
# Hand-off precision and layout of the large tensor
# --------------------------------------------------------------------------------------

def large_to_token_major(t_l: np.ndarray, n_tok: int, j2: int, i1: int = 1) -> np.ndarray:
    """T_L[r, (a2, b2)] -> K'[a2*i1 + rho, r'*j2 + b2] with r = rho*j1 + r', rounded to fp32 (the
    precision the quantizer sees).  n_tok = i1 * i2 rows of d = j1*j2 elements: with i1 = 1 row t
    is token t; with i1 > 1 the i1 rows a2*i1 + rho hold the i1 slices of the bond index that
    belong to position a2, so the row count and the row length are those of the block itself."""
    i2 = n_tok // i1
    j1 = t_l.shape[0] // i1
    return np.ascontiguousarray(
        t_l.reshape(i1, j1, i2, j2).transpose(2, 0, 1, 3).reshape(i2 * i1, j1 * j2)).astype(np.float32)


def token_major_to_large(kp: np.ndarray, j1: int, j2: int, i1: int = 1) -> np.ndarray:
    """Inverse layout change of `large_to_token_major` (values untouched)."""
    i2 = kp.shape[0] // i1
    return kp.reshape(i2, i1, j1, j2).transpose(1, 2, 0, 3).reshape(i1 * j1, i2 * j2)


# --------------------------------------------------------------------------------------
# Eq. 1 per group: step, code, dequantized value
# --------------------------------------------------------------------------------------

def group_steps(kp: np.ndarray, group: int, qmax: int, full_range: bool = False) -> np.ndarray:
    """Delta[t, g] = fp16(max|x| over group / qmax), the quotient rounded once to fp16.

    The fp64 quotient of a 24-bit numerator by qmax <= 127 cannot land within
    fp64 rounding distance of an fp16 rounding boundary without being on it, so
    fp64-divide-then-cast equals a single rounding of the exact quotient.

    full_range (codes [-qmax - 1, qmax]): the smallest step under which neither end clips,
    Delta = fp16(max(max(x) / qmax, max(-x) / (qmax + 1))); rounding is monotonic, so the larger of
    the two rounded quotients is the rounded larger quotient.
    """
    n_tok, d = kp.shape
    x = kp.astype(np.float64).reshape(n_tok, d // group, group)
    with np.errstate(over="ignore"):
        if not full_range:
            return (np.abs(x).max(axis=2) / float(qmax)).astype(np.float16)
        up = (np.maximum(x, 0.0).max(axis=2) / float(qmax)).astype(np.float16)
        down = (np.maximum(-x, 0.0).max(axis=2) / float(qmax + 1)).astype(np.float16)
        return np.maximum(up, down)


def quantize_codes(kp: np.ndarray, steps: np.ndarray, group: int, qmax: int, full_range: bool = False) -> np.ndarray:
    """c[t, e] = clamp(round_half_even(x / Delta), lo, qmax), lo = -qmax (or -qmax - 1 with
    full_range); all-zero where Delta == 0."""
    n_tok, d = kp.shape
    delta = np.repeat(steps.astype(np.float64), group, axis=1)
    x = kp.astype(np.float64)
    safe = np.where(delta > 0, delta, 1.0)
    c = np.rint(x / safe)
    c = np.clip(c, -qmax - (1 if full_range else 0), qmax)
    c = np.where(delta > 0, c, 0.0)
    return c.astype(np.int32)


def dequantize(codes: np.ndarray, steps: np.ndarray, group: int) -> np.ndarray:
    """x_hat[t, e] = Delta[t, group(e)] * c[t, e] in fp64 (exact: 11-bit x 8-bit product)."""
    return np.repeat(steps.astype(np.float64), group, axis=1) * codes.astype(np.float64)


def rtn_whole_matrix(w: np.ndarray, bits: int) -> np.ndarray:
    """Eq. 1 as printed, one step for the whole matrix: returns the dequantized matrix
    Delta * round(W / Delta), Delta = max|W| / (2^(bits-1) - 1), in fp64 (no fp16 step here)."""
    qmax = (1 << (bits - 1)) - 1
    a = np.abs(w).max()
    if a == 0:
        return np.zeros_like(w, dtype=np.float64)
    delta = a / qmax
    return delta * np.clip(np.rint(w / delta), -qmax, qmax)


# --------------------------------------------------------------------------------------
# Bit packing of codes (storage format)
# --------------------------------------------------------------------------------------

def pack_rows(codes: np.ndarray, bits: int) -> np.ndarray:
    """Pack signed codes along the last axis, offset-binary, little-endian within a byte.

    Stored field u = c + 2^(bits-1).  Element e of a row occupies bits
    [(e*bits) % 8, (e*bits) % 8 + bits) of byte (e*bits) // 8.
    """
    u = (codes.astype(np.int64) + (1 << (bits - 1))).astype(np.uint8)
    per = 8 // bits
    shape = u.shape[:-1] + (u.shape[-1] // per, per)
    u = u.reshape(shape)
    out = np.zeros(shape[:-1], np.uint8)
    for k in range(per):
        out |= (u[..., k] << (k * bits)).astype(np.uint8)
    return out


def unpack_rows(packed: np.ndarray, bits: int) -> np.ndarray:
    """Inverse of `pack_rows`: returns signed int32 codes."""
    per = 8 // bits
    mask = (1 << bits) - 1
    fields = [((packed >> (k * bits)) & mask).astype(np.int32) for k in range(per)]
    u = np.stack(fields, axis=-1).reshape(packed.shape[:-1] + (packed.shape[-1] * per,))
    return u - (1 << (bits - 1))


def value_codes_to_tiles(codes: np.ndarray, j1: int, j2: int) -> np.ndarray:
    """Reorder value codes c[t, r*j2 + b2] of one block to [tile, b2, r, token-in-tile].

    Value codes are stored so that the tokens of one large-tensor row are
    contiguous (the contraction P.V' runs over tokens).
    """
    n_tok = codes.shape[0]
    n_tiles = n_tok // TILE_TOKENS
    c = codes.reshape(n_tiles, TILE_TOKENS, j1, j2)
    return np.ascontiguousarray(c.transpose(0, 3, 2, 1))


def value_tiles_to_codes(tiles: np.ndarray) -> np.ndarray:
    """Inverse of `value_codes_to_tiles`: [tile, b2, r, tok] -> c[t, r*j2 + b2]."""
    n_tiles, j2, j1, tt = tiles.shape
    return np.ascontiguousarray(tiles.transpose(0, 3, 2, 1)).reshape(n_tiles * tt, j1 * j2)


# --------------------------------------------------------------------------------------
# One block: compress, reconstruct
# --------------------------------------------------------------------------------------

@dataclass
class Block:
    """One compressed [block_tokens, head_dim] block of keys or of values (natural layouts)."""
    small: np.ndarray    # fp16 [j1 (b1), j1 (r)]   T_S  (i1 > 1: [i1*j1 (a1, b1), i1*j1 (r)])
    steps: np.ndarray    # fp16 [block_tokens, head_dim/group]
    codes: np.ndarray    # int32 [block_tokens, head_dim], element index r*j2 + b2
    large32: np.ndarray  # fp32 [block_tokens, head_dim], the unquantized large tensor, token-major
    small3: Optional[np.ndarray] = None   # fp16 [i3 (bond e), i3 (token a3)]   T_3, three tensors
                                          # (four: [i3*i4 (bond e), i3 (token a3), i4 (bond f)])
    small4: Optional[np.ndarray] = None   # fp16 [i4 (bond f), i4 (token a4)]   T_4, four tensors only


def compress_block(x: np.ndarray, fmt: Format, n_valid: Optional[int] = None,
                   sigma_in: str = "small", identity_small: bool = False) -> Block:
    """DecoQuant of one block (Section 3.1): decompose, quantize T_L, keep T_S in fp16.

    x: fp16 (or any float) [<= block_tokens, head_dim]; rows >= n_valid and missing
    rows are zero.  identity_small=True skips the decomposition (T_S = I), which is
    plain group round-to-nearest on the block.
    """
    fmt.check()
    tb, d = fmt.block_tokens, fmt.head_dim
    n = x.shape[0] if n_valid is None else n_valid
    xb = np.zeros((tb, d), np.float64)
    xb[:n] = np.asarray(x[:n], dtype=np.float64)
    small3 = small4 = None
    if fmt.i3 > 1:
        if identity_small or sigma_in != "small":
            raise ValueError("the three- and four-tensor forms have no identity / sigma-in-large variant")
        if fmt.i4 > 1:
            t_s, t_2, t_3, t_4 = mpo4_split(xb, fmt.j1, fmt.i3, fmt.i4)
        else:
            t_s, t_2, t_3 = mpo3_split(xb, fmt.j1, fmt.i3)
        kp = middle_to_token_major(t_2)
        with np.errstate(over="ignore"):
            small3 = t_3.astype(np.float16)
            if fmt.i4 > 1:
                small4 = t_4.astype(np.float16)
    else:
        if identity_small:
            t_s = np.eye(fmt.small_side)
            t_l = matricise(xb, fmt.i1, fmt.j1)
        else:
            t_s, t_l = mpo_split(xb, fmt.j1, fmt.i1, sigma_in)
        kp = large_to_token_major(t_l, tb, fmt.j2, fmt.i1)
    steps = group_steps(kp, fmt.group, fmt.qmax, fmt.full_range)
    codes = quantize_codes(kp, steps, fmt.group, fmt.qmax, fmt.full_range)
    with np.errstate(over="ignore"):
        small = t_s.astype(np.float16)
    return Block(small=small, steps=steps, codes=codes, large32=kp, small3=small3, small4=small4)


def _token_factor(small3: np.ndarray, small4: Optional[np.ndarray], fmt: Format, absolute: bool = False) -> np.ndarray:
    """What multiplies the middle tensor on the token side, as one matrix [bond e, token in run]:
    T_3 itself (three tensors), or T_3 contracted with T_4 over the bond f (four; token (a3, a4)).
    absolute: the same with every entry replaced by its magnitude (for error bounds)."""
    t_3 = small3.astype(np.float64)
    if fmt.i4 == 1:
        return np.abs(t_3) if absolute else t_3
    t_4 = small4.astype(np.float64)
    if absolute:
        t_3, t_4 = np.abs(t_3), np.abs(t_4)
    return np.einsum("def,fg->deg", t_3, t_4).reshape(fmt.bond3, fmt.bond3)


def reconstruct_block(small: np.ndarray, steps: np.ndarray, codes: np.ndarray, fmt: Format,
                      small3: Optional[np.ndarray] = None, small4: Optional[np.ndarray] = None) -> np.ndarray:
    """X_hat[block_tokens, head_dim] = un-matricise(T_S16 @ (Delta * c)) in fp64, no rounding.
    Three tensors: the dequantized middle tensor is first multiplied by T_3 (fp16 values) over
    the bond e, which gives the right factor of the first cut back; four: by T_3 and T_4."""
    # rows past the valid tokens of a partly filled block may hold anything (NaN steps included)
    with np.errstate(invalid="ignore", over="ignore"):
        deq = dequantize(codes, steps, fmt.group)
        if fmt.i3 > 1:
            t_2_hat = token_major_to_middle(deq, fmt.j1, fmt.j2, fmt.bond3)       # [r, a2, b2, e]
            right = np.einsum("racd,de->raec", t_2_hat, _token_factor(small3, small4, fmt))  # [r, a2, token in run, b2]
            t_l_hat = right.reshape(fmt.j1, fmt.block_tokens * fmt.j2)
        else:
            t_l_hat = token_major_to_large(deq, fmt.j1, fmt.j2, fmt.i1)
        m_hat = small.astype(np.float64) @ t_l_hat
    return unmatricise(m_hat, fmt.block_tokens, fmt.head_dim, fmt.i1, fmt.j1)


def reconstruction_bound(small: np.ndarray, steps: np.ndarray, fmt: Format,
                         small3: Optional[np.ndarray] = None, small4: Optional[np.ndarray] = None) -> np.ndarray:
    """Elementwise bound on |X_hat - T_S16 @ T_L| from the Delta/2 code error:
    0.5 * sum_r |T_S16[b1, r]| * Delta[t, group(r*j2 + b2)], shape [block_tokens, head_dim].
    Three tensors: Delta[t, .] is replaced by sum_e |T_3[e, a3]| * Delta[(a2, e), .]; four: by the
    same sum with sum_f |T_3[e, a3, f]| |T_4[f, a4]| in the place of |T_3[e, a3]|."""
    tb, d = fmt.block_tokens, fmt.head_dim
    delta = np.repeat(steps.astype(np.float64), fmt.group, axis=1)      # [t, r*j2+b2]
    if fmt.i3 > 1:
        dm = token_major_to_middle(delta, fmt.j1, fmt.j2, fmt.bond3)    # [r, a2, b2, e]
        right = np.einsum("racd,de->raec", dm, _token_factor(small3, small4, fmt, absolute=True))
        delta_l = right.reshape(fmt.j1, tb * fmt.j2)
    else:
        delta_l = token_major_to_large(delta, fmt.j1, fmt.j2, fmt.i1)   # [r, (a2, b2)]
    m_bound = 0.5 * np.abs(small.astype(np.float64)) @ delta_l
    return unmatricise(m_bound, tb, d, fmt.i1, fmt.j1)


# --------------------------------------------------------------------------------------
# Whole cache in the storage layout the library reads
# --------------------------------------------------------------------------------------

def empty_cache(fmt: Format, batch: int, kv_heads: int, block_capacity: int) -> Dict[str, np.ndarray]:
    """Zero-filled arrays with the storage layout:
      k_codes  u8  [B, H, NB, T_b, d*bits/8]              token-major rows
      k_scales f16 [B, H, NB, T_b, d/G]
      k_small  f16 [B, H, NB, j1 (r), j1 (b1)]             T_S of keys, TRANSPOSED (bond index first)
                                                           (i1 > 1: both sides i1*j1, rows (a1, b1))
      v_codes  u8  [B, H, NB, T_b/128, j2, j1, 128*bits/8] token-contiguous inside 128-token tiles
      v_scales f16 [B, H, NB, T_b, d/G]
      v_small  f16 [B, H, NB, j1 (b1), j1 (r)]             T_S of values, natural
    and, with three local tensors,
      k_small3 f16 [B, H, NB, i3 (token a3), i3 (bond e)]  T_3 of keys, TRANSPOSED (token first)
      v_small3 f16 [B, H, NB, i3 (bond e), i3 (token a3)]  T_3 of values, natural
    and, with four (this module's own arrangement: no library reads it), both T_3 natural and flat,
      k_small3, v_small3 f16 [B, H, NB, i3*i4 (bond e), i3*i4 ((a3, f))]
      k_small4, v_small4 f16 [B, H, NB, i4 (bond f), i4 (token a4)]
    """
    fmt.check()
    b, h, nb, tb, d = batch, kv_heads, block_capacity, fmt.block_tokens, fmt.head_dim
    tiles = tb // TILE_TOKENS
    extra = {}
    if fmt.i3 > 1:
        extra = {"k_small3": np.zeros((b, h, nb, fmt.bond3, fmt.bond3), np.float16),
                 "v_small3": np.zeros((b, h, nb, fmt.bond3, fmt.bond3), np.float16)}
    if fmt.i4 > 1:
        extra["k_small4"] = np.zeros((b, h, nb, fmt.i4, fmt.i4), np.float16)
        extra["v_small4"] = np.zeros((b, h, nb, fmt.i4, fmt.i4), np.float16)
    return {
        **extra,
        "k_codes": np.zeros((b, h, nb, tb, fmt.row_bytes), np.uint8),
        "k_scales": np.zeros((b, h, nb, tb, fmt.groups_per_row), np.float16),
        "k_small": np.zeros((b, h, nb, fmt.small_side, fmt.small_side), np.float16),
        "v_codes": np.zeros((b, h, nb, tiles, fmt.j2, fmt.j1, TILE_TOKENS * fmt.bits // 8), np.uint8),
        "v_scales": np.zeros((b, h, nb, tb, fmt.groups_per_row), np.float16),
        "v_small": np.zeros((b, h, nb, fmt.small_side, fmt.small_side), np.float16),
    }


def store_block(cache: Dict[str, np.ndarray], fmt: Format, b: int, h: int, blk: int,
                kblock: Block, vblock: Block) -> None:
    """Write one compressed key block and value block into the storage arrays."""
    cache["k_codes"][b, h, blk] = pack_rows(kblock.codes, fmt.bits)
    cache["k_scales"][b, h, blk] = kblock.steps
    cache["k_small"][b, h, blk] = kblock.small.T
    cache["v_codes"][b, h, blk] = pack_rows(value_codes_to_tiles(vblock.codes, fmt.j1, fmt.j2), fmt.bits)
    cache["v_scales"][b, h, blk] = vblock.steps
    cache["v_small"][b, h, blk] = vblock.small
    if fmt.i4 > 1:
        for name, blk_ in (("k", kblock), ("v", vblock)):
            cache[name + "_small3"][b, h, blk] = blk_.small3.reshape(fmt.bond3, fmt.bond3)
            cache[name + "_small4"][b, h, blk] = blk_.small4
    elif fmt.i3 > 1:
        cache["k_small3"][b, h, blk] = kblock.small3.T
        cache["v_small3"][b, h, blk] = vblock.small3


def load_block(cache: Dict[str, np.ndarray], fmt: Format, b: int, h: int, blk: int, which: str
               ) -> Tuple:
    """Read (small [b1, r] fp16, steps, signed codes [t, r*j2+b2]) of a key ('k') or value ('v')
    block; with three local tensors a fourth item, T_3 [e, a3] fp16, follows; with four, T_3
    [e, a3, f] and T_4 [f, a4]."""
    if fmt.i4 > 1:
        if which == "k":
            codes = unpack_rows(cache["k_codes"][b, h, blk], fmt.bits)
            first = (cache["k_small"][b, h, blk].T, cache["k_scales"][b, h, blk], codes)
        else:
            codes = value_tiles_to_codes(unpack_rows(cache["v_codes"][b, h, blk], fmt.bits))
            first = (cache["v_small"][b, h, blk], cache["v_scales"][b, h, blk], codes)
        return first + (cache[which + "_small3"][b, h, blk].reshape(fmt.bond3, fmt.i3, fmt.i4),
                        cache[which + "_small4"][b, h, blk])
    if which == "k":
        codes = unpack_rows(cache["k_codes"][b, h, blk], fmt.bits)
        out = (cache["k_small"][b, h, blk].T, cache["k_scales"][b, h, blk], codes)
        return out + ((cache["k_small3"][b, h, blk].T,) if fmt.i3 > 1 else ())
    codes = value_tiles_to_codes(unpack_rows(cache["v_codes"][b, h, blk], fmt.bits))
    out = (cache["v_small"][b, h, blk], cache["v_scales"][b, h, blk], codes)
    return out + ((cache["v_small3"][b, h, blk],) if fmt.i3 > 1 else ())


def compress_sequence(cache: Dict[str, np.ndarray], fmt: Format, b: int, h: int,
                      k: np.ndarray, v: np.ndarray, first_block: int = 0,
                      identity_small: bool = False) -> None:
    """Compress K, V [n_tok, d] of one (sequence, kv head) block by block (Section 3.2)."""
    n_tok = k.shape[0]
    tb = fmt.block_tokens
    for i, t0 in enumerate(range(0, n_tok, tb)):
        kb = compress_block(k[t0:t0 + tb], fmt, identity_small=identity_small)
        vb = compress_block(v[t0:t0 + tb], fmt, identity_small=identity_small)
        store_block(cache, fmt, b, h, first_block + i, kb, vb)


def reconstruct_sequence(cache: Dict[str, np.ndarray], fmt: Format, b: int, h: int, n_tok: int
                         ) -> Tuple[np.ndarray, np.ndarray]:
    """Dequantized K_hat, V_hat [n_tok, d] in fp64 for one (sequence, kv head)."""
    tb, d = fmt.block_tokens, fmt.head_dim
    n_blk = -(-n_tok // tb)
    k_hat = np.zeros((n_blk * tb, d))
    v_hat = np.zeros((n_blk * tb, d))
    for blk in range(n_blk):
        kb, vb = load_block(cache, fmt, b, h, blk, "k"), load_block(cache, fmt, b, h, blk, "v")
        k_hat[blk * tb:(blk + 1) * tb] = reconstruct_block(kb[0], kb[1], kb[2], fmt, *kb[3:])
        v_hat[blk * tb:(blk + 1) * tb] = reconstruct_block(vb[0], vb[1], vb[2], fmt, *vb[3:])
    return k_hat[:n_tok], v_hat[:n_tok]


# --------------------------------------------------------------------------------------
# Attention
# --------------------------------------------------------------------------------------

def dense_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: Optional[float] = None
                    ) -> np.ndarray:
    """softmax(q K^T * scale) V for one query row, fp64, max-subtracted.  Empty K -> zeros."""
    d = q.shape[-1]
    if k.shape[0] == 0:
        return np.zeros(v.shape[-1])
    sc = (1.0 / np.sqrt(d)) if scale is None else scale
    s = (k.astype(np.float64) @ q.astype(np.float64)) * sc
    p = np.exp(s - s.max())
    p /= p.sum()
    return p @ v.astype(np.float64)


def attention_decode(cache: Dict[str, np.ndarray], fmt: Format, q: np.ndarray, seq_lens: np.ndarray,
                     scale: Optional[float] = None,
                     pairs: Optional[Sequence[Tuple[int, int]]] = None,
                     k_tail: Optional[np.ndarray] = None, v_tail: Optional[np.ndarray] = None,
                     tail_lens: Optional[np.ndarray] = None) -> np.ndarray:
    """Decode-step attention against the compressed cache (Section 3.2): dequantize the
    blocks of each (sequence, kv head) and run ordinary attention for every query head
    mapped to that kv head (h_kv = h_q // (H_q / H_kv)).

    q: fp16 [B, H_q, d]; returns fp64 [B, H_q, d].  With `pairs`, only the listed
    (b, h_kv) pairs are computed; other rows stay NaN.

    k_tail, v_tail [B, H_kv, cap, d] with tail_lens [B]: the tokens generated since the last
    compression, still held in fp16 (Section 3.2: new rows are buffered and DecoQuant runs only
    when a block's worth has accumulated).  They follow the compressed tokens and are attended
    to at full precision.
    """
    bsz, hq, d = q.shape
    hkv = cache["k_codes"].shape[1]
    rep = hq // hkv
    out = np.full((bsz, hq, d), np.nan)
    todo = pairs if pairs is not None else [(b, h) for b in range(bsz) for h in range(hkv)]
    for b, h in todo:
        n_tok = int(seq_lens[b])
        k_hat, v_hat = reconstruct_sequence(cache, fmt, b, h, n_tok)
        if k_tail is not None:
            n_tail = int(tail_lens[b])
            k_hat = np.concatenate([k_hat, k_tail[b, h, :n_tail].astype(np.float64)])
            v_hat = np.concatenate([v_hat, v_tail[b, h, :n_tail].astype(np.float64)])
        for hq_i in range(h * rep, (h + 1) * rep):
            out[b, hq_i] = dense_attention(q[b, hq_i], k_hat, v_hat, scale)
    return out


# --------------------------------------------------------------------------------------
# Eq. 4: compression ratio
# --------------------------------------------------------------------------------------

def compression_ratio(fmt: Format, step_bits: int = 16) -> float:
    """mu = (#T_L * B + #T_S * 16 + bits of the steps) / (#W * 16) for one block (Eq. 4)."""
    n_w = fmt.block_tokens * fmt.head_dim
    n_l = fmt.j1 * fmt.block_tokens * fmt.j2
    n_s = fmt.small_side * fmt.small_side + (fmt.bond3 * fmt.bond3 if fmt.i3 > 1 else 0) + (fmt.i4 * fmt.i4 if fmt.i4 > 1 else 0)
    n_delta = fmt.block_tokens * fmt.groups_per_row
    return (n_l * fmt.bits + n_s * 16 + n_delta * step_bits) / (n_w * 16.0)


def cache_bytes_per_block(fmt: Format) -> int:
    """Bytes one key (or value) block occupies in the storage arrays."""
    return (fmt.block_tokens * fmt.row_bytes + fmt.block_tokens * fmt.groups_per_row * 2
            + fmt.small_side * fmt.small_side * 2 + (fmt.bond3 * fmt.bond3 * 2 if fmt.i3 > 1 else 0)
            + (fmt.i4 * fmt.i4 * 2 if fmt.i4 > 1 else 0))
