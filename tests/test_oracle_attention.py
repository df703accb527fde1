"""Pins for the oracle's block reconstruction and decode attention (Sections 3.1-3.2)."""
import numpy as np
import pytest

from oracle import decoquant_oracle as O
import workloads


def _outlier_block(seed, n_tok=128, d=128, n_out=4, scale=20.0, token_scale=True):
    r = np.random.default_rng(seed)
    x = r.standard_normal((n_tok, d))
    if token_scale:
        x *= np.exp(0.5 * r.standard_normal((n_tok, 1)))
    x[:, r.choice(d, n_out, replace=False)] *= scale
    return x.astype(np.float16)


def test_reconstruction_error_within_the_half_step_bound():
    fmt = O.Format(4, 128, 128, 16, 8, 128)
    x = _outlier_block(1)
    blk = O.compress_block(x, fmt)
    x_hat = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt)
    bound = O.reconstruction_bound(blk.small, blk.steps, fmt)
    # plus fp16 rounding of T_S and fp32 rounding of T_L (relative 2^-11 and 2^-24 per term)
    t_l = O.token_major_to_large(blk.large32.astype(np.float64), 16, 8)
    slack = O.unmatricise(2.0 ** -11 * np.abs(blk.small.astype(np.float64)) @ np.abs(t_l), 128, 128, 1, 16)
    err = np.abs(x_hat - x.astype(np.float64))
    assert (err <= bound + slack + 1e-9).all()
    assert err.max() > 1e-3          # it is a lossy code, the bound is not vacuous
    # a transposed small tensor breaks it: the pin is sensitive to index order
    wrong = O.reconstruct_block(blk.small.T.copy(), blk.steps, blk.codes, fmt)
    assert not (np.abs(wrong - x.astype(np.float64)) <= bound + slack + 1e-9).all()


@pytest.mark.parametrize("fmt", [O.Format(4, 128, 128, 16, 8, 128), O.Format(4, 64, 64, 8, 8, 256)])
def test_decoquant_beats_plain_rtn_on_outlier_blocks(fmt):
    # Section 4.3 "Effectiveness of Tensor Quantization": quantizing only T_L gives a lower
    # reconstruction error than quantizing the matrix itself (direction only).
    wins = 0
    for seed in range(4):
        x = _outlier_block(20 + seed, fmt.block_tokens, fmt.head_dim, 4 if fmt.head_dim == 128 else 2,
                           token_scale=False)
        dq = O.compress_block(x, fmt)
        rtn = O.compress_block(x, fmt, identity_small=True)
        e_dq = np.linalg.norm(O.reconstruct_block(dq.small, dq.steps, dq.codes, fmt) - x.astype(np.float64))
        e_rtn = np.linalg.norm(O.reconstruct_block(rtn.small, rtn.steps, rtn.codes, fmt) - x.astype(np.float64))
        wins += e_dq < e_rtn
    assert wins == 4


def test_identity_small_tensor_is_plain_group_rtn():
    fmt = O.Format(4, 64, 128, 16, 8, 128)
    x = _outlier_block(2)
    blk = O.compress_block(x, fmt, identity_small=True)
    # with T_S = I the large tensor in token-major order is the block itself
    assert np.array_equal(blk.large32, x.astype(np.float32))
    xf = x.astype(np.float64)
    for t in (0, 5, 127):
        for g in range(2):
            seg = xf[t, g * 64:(g + 1) * 64]
            step = np.float16(np.abs(seg).max() / 7)
            assert blk.steps[t, g] == step
            want = np.clip(np.rint(seg / float(step)), -7, 7)
            assert np.array_equal(blk.codes[t, g * 64:(g + 1) * 64], want)
    x_hat = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt)
    assert np.array_equal(x_hat, O.dequantize(blk.codes, blk.steps, 64))


def _lossless_kv(seed, n_tok, d, qmax):
    """Blocks that identity-small group quantization represents exactly."""
    r = np.random.default_rng(seed)
    c = r.integers(-qmax, qmax + 1, size=(n_tok, d))
    c[:, 0] = qmax                          # every row's group max is qmax * step
    c[:, d // 2] = -qmax
    step = 2.0 ** r.integers(-4, 1, size=(n_tok, 1))
    return (c * step).astype(np.float16)


def test_attention_equals_dense_attention_when_the_code_is_lossless():
    # T_S = I and exactly representable rows: the whole storage path (pack, tile layout,
    # load, dequantize, GQA head map, masking) must reproduce brute-force dense attention.
    fmt = O.Format(4, 64, 128, 16, 8, 128)
    bsz, hq, hkv, n_tok = 2, 4, 2, 300
    cache = O.empty_cache(fmt, bsz, hkv, 3)
    r = np.random.default_rng(5)
    ks, vs = {}, {}
    for b in range(bsz):
        for h in range(hkv):
            ks[b, h] = _lossless_kv(10 * b + h, n_tok, 128, 7)
            vs[b, h] = _lossless_kv(100 + 10 * b + h, n_tok, 128, 7)
            O.compress_sequence(cache, fmt, b, h, ks[b, h], vs[b, h], identity_small=True)
    q = r.standard_normal((bsz, hq, 128)).astype(np.float16)
    lens = np.array([300, 129], np.int32)
    out = O.attention_decode(cache, fmt, q, lens)
    for b in range(bsz):
        for i in range(hq):
            h = i // 2
            want = O.dense_attention(q[b, i], ks[b, h][:lens[b]], vs[b, h][:lens[b]])
            assert np.abs(out[b, i] - want).max() <= 1e-10


def test_unquantized_decomposition_gives_dense_attention():
    # Exact MPO (no quantization): attention on T_S x T_L equals attention on the matrix.
    x_k, x_v = _outlier_block(3).astype(np.float64), _outlier_block(4).astype(np.float64)
    rec = []
    for x in (x_k, x_v):
        t_s, t_l = O.mpo_split(x, 16)
        rec.append(O.unmatricise(t_s @ t_l, 128, 128, 1, 16))
    q = np.random.default_rng(0).standard_normal(128)
    assert np.abs(O.dense_attention(q, rec[0], rec[1]) - O.dense_attention(q, x_k, x_v)).max() <= 1e-10


def test_dense_attention_against_explicit_loops():
    r = np.random.default_rng(8)
    q, k, v = r.standard_normal(16), r.standard_normal((9, 16)), r.standard_normal((9, 16))
    s = [sum(q[c] * k[t, c] for c in range(16)) / 4.0 for t in range(9)]
    w = [np.exp(x) for x in s]
    want = [sum(w[t] * v[t, c] for t in range(9)) / sum(w) for c in range(16)]
    assert np.allclose(O.dense_attention(q, k, v), want, atol=1e-12)


def test_softmax_invariants_on_the_quantized_path():
    w = workloads.get_workload("tiny")
    fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens)
    cache = O.empty_cache(fmt, 1, w.kv_heads, 1)
    for h in range(w.kv_heads):
        k, v = workloads.kv_pair(w, 0, h)
        O.compress_sequence(cache, fmt, 0, h, k, v)
    q = workloads.query(w)
    # one cached token: the output is that token's dequantized value row
    out1 = O.attention_decode(cache, fmt, q, np.array([1], np.int32))
    for h in range(w.kv_heads):
        _, v_hat = O.reconstruct_sequence(cache, fmt, 0, h, 1)
        assert np.abs(out1[0, h] - v_hat[0]).max() <= 1e-12
    # empty sequence: zeros
    assert (O.attention_decode(cache, fmt, q, np.array([0], np.int32)) == 0).all()
    # convex combination: every output channel lies between the extremes of V_hat
    out = O.attention_decode(cache, fmt, q, np.array([200], np.int32))
    for h in range(w.kv_heads):
        _, v_hat = O.reconstruct_sequence(cache, fmt, 0, h, 200)
        assert (out[0, h] <= v_hat.max(axis=0) + 1e-12).all()
        assert (out[0, h] >= v_hat.min(axis=0) - 1e-12).all()
    # close to attention on the original fp16 K, V (the code is lossy but small at 4 bits)
    for h in range(w.kv_heads):
        k, v = workloads.kv_pair(w, 0, h, 200)
        ref = O.dense_attention(q[0, h], k, v)
        assert np.abs(out[0, h] - ref).max() < 0.1 * np.abs(v.astype(np.float64)).max()


def test_pairs_argument_restricts_the_work():
    w = workloads.get_workload("tiny")
    fmt = O.Format(w.bits, w.group, w.head_dim, w.j1, w.j2, w.block_tokens)
    cache = O.empty_cache(fmt, 1, w.kv_heads, 1)
    k, v = workloads.kv_pair(w, 0, 2)
    O.compress_sequence(cache, fmt, 0, 2, k, v)
    out = O.attention_decode(cache, fmt, workloads.query(w), workloads.seq_lens(w), pairs=[(0, 2)])
    assert np.isfinite(out[0, 2]).all() and np.isnan(out[0, 0]).all()


def test_fp16_tail_is_attended_like_extra_tokens():
    # Section 3.2: rows generated since the last compression stay in fp16.  With a lossless code
    # the result must equal brute-force dense attention over [compressed tokens, tail tokens];
    # an empty tail changes nothing; a tail alone (no compressed token) is plain attention.
    fmt = O.Format(4, 64, 128, 16, 8, 128)
    r = np.random.default_rng(11)
    k, v = _lossless_kv(1, 200, 128, 7), _lossless_kv(2, 200, 128, 7)
    cache = O.empty_cache(fmt, 2, 1, 2)
    for b in range(2):
        O.compress_sequence(cache, fmt, b, 0, k, v, identity_small=True)
    kt = r.standard_normal((2, 1, 16, 128)).astype(np.float16)
    vt = r.standard_normal((2, 1, 16, 128)).astype(np.float16)
    q = r.standard_normal((2, 2, 128)).astype(np.float16)
    lens, tl = np.array([200, 0], np.int32), np.array([5, 16], np.int32)
    out = O.attention_decode(cache, fmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=tl)
    for hq in range(2):
        want = O.dense_attention(q[0, hq], np.concatenate([k[:200], kt[0, 0, :5]]), np.concatenate([v[:200], vt[0, 0, :5]]))
        assert np.abs(out[0, hq] - want).max() <= 1e-10
        want = O.dense_attention(q[1, hq], kt[1, 0], vt[1, 0])
        assert np.abs(out[1, hq] - want).max() <= 1e-10
    none = O.attention_decode(cache, fmt, q, lens, k_tail=kt, v_tail=vt, tail_lens=np.zeros(2, np.int32))
    base = O.attention_decode(cache, fmt, q, lens)
    assert np.array_equal(none, base)


def test_quantization_strategy_ordering_on_outlier_blocks():
    # Section 4.3 "Effectiveness of Tensor Quantization": quantizing only T_L gives the lowest
    # reconstruction error, quantizing both local tensors is worse, quantizing the matrix itself
    # is worst.  Same granularity for all three (one step per group of a token row; T_S, when
    # quantized, gets one step for the whole small tensor as in Eq. 1).  Direction only.
    fmt = O.Format(4, 128, 128, 16, 8, 128)
    rows = []
    for seed in range(4):
        x = _outlier_block(40 + seed, token_scale=False).astype(np.float64)
        dq = O.compress_block(x, fmt)
        only_large = np.linalg.norm(O.reconstruct_block(dq.small, dq.steps, dq.codes, fmt) - x)
        t_l_hat = O.token_major_to_large(O.dequantize(dq.codes, dq.steps, fmt.group), 16, 8)
        t_s_q = O.rtn_whole_matrix(dq.small.astype(np.float64), 4)
        both = np.linalg.norm(O.unmatricise(t_s_q @ t_l_hat, 128, 128, 1, 16) - x)
        rtn = O.compress_block(x, fmt, identity_small=True)
        matrix = np.linalg.norm(O.reconstruct_block(rtn.small, rtn.steps, rtn.codes, fmt) - x)
        rows.append((only_large, both, matrix))
        assert only_large < both
        assert only_large < matrix
    # the middle variant is reported, not asserted against the matrix variant: with a 4-bit small
    # tensor the singular values themselves are rounded, which on these blocks costs more than the
    # outliers do (the paper's figure has the opposite order on LLaMA activations)
    print("reconstruction error (T_L only, both, matrix):", [tuple(round(v, 1) for v in r) for r in rows])


def test_rtn_whole_matrix_is_eq1():
    w = np.array([[0.5, -3.0], [1.49, 2.26]])
    got = O.rtn_whole_matrix(w, 3)            # qmax = 3, Delta = 1: round to integers
    assert np.array_equal(got, np.array([[0.0, -3.0], [1.0, 2.0]]))
