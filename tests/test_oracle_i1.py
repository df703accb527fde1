"""Pins for the oracle's i_1 > 1 factor shapes (Preliminary, Eq. 2 with n = 2 and a token factor on
the small tensor): X[(a1, a2), (b1, b2)] = sum_r T_S[(a1, b1), r] T_L[r, (a2, b2)]."""
import numpy as np
import pytest

from oracle import decoquant_oracle as O


def _block(seed, n_tok=128, d=128, outliers=(3, 40, 77, 100), scale=20.0):
    r = np.random.default_rng(seed)
    x = r.standard_normal((n_tok, d))
    x[:, list(outliers)] *= scale
    return x.astype(np.float16)


def test_row_layout_of_the_large_tensor_against_explicit_loops():
    i1, i2, j1, j2 = 2, 3, 4, 5
    t_l = np.arange(i1 * j1 * i2 * j2, dtype=np.float64).reshape(i1 * j1, i2 * j2)
    kp = O.large_to_token_major(t_l, i1 * i2, j2, i1)
    assert kp.shape == (i1 * i2, j1 * j2) and kp.dtype == np.float32
    for rho in range(i1):
        for rp in range(j1):
            for a2 in range(i2):
                for b2 in range(j2):
                    assert kp[a2 * i1 + rho, rp * j2 + b2] == t_l[rho * j1 + rp, a2 * j2 + b2]
    assert np.array_equal(O.token_major_to_large(kp.astype(np.float64), j1, j2, i1), t_l)
    # i1 = 1 is the plain token-major layout: row t holds T_L[:, (t, :)]
    plain = O.large_to_token_major(t_l, (i2 * j2) // j2, j2, 1)
    assert np.array_equal(plain[1], t_l[:, j2:2 * j2].reshape(-1).astype(np.float32))


@pytest.mark.parametrize("i1,j1,d,tb", [(2, 16, 128, 128), (4, 8, 128, 256), (2, 8, 64, 128), (2, 4, 64, 128)])
def test_split_with_a_token_factor_is_exact_and_agrees_with_the_general_routine(i1, j1, d, tb):
    x = _block(3, tb, d, outliers=(1, 9)).astype(np.float64)
    t_s, t_l = O.mpo_split(x, j1, i1)
    n = i1 * j1
    i2, j2 = tb // i1, d // j1
    assert t_s.shape == (n, n) and t_l.shape == (n, i2 * j2)
    m = O.matricise(x, i1, j1)
    assert np.linalg.norm(t_s @ t_l - m) / np.linalg.norm(m) <= 1e-10
    assert np.abs(t_l @ t_l.T - np.eye(n)).max() <= 1e-12
    assert t_s.size + t_l.size == x.size + n * n           # a few more parameters than the matrix (Section 3.3)
    # the two factors, viewed as the 4-index local tensors of Eq. 2, multiply back to X term by term
    back = O.mpo_contract(O.as_local_tensors(t_s, t_l, i1, j1, i2, j2))
    assert np.abs(back - x).max() <= 1e-9
    # and the general n-site routine finds the same product with the same shapes
    tens = O.mpo_decompose(x, (i1, i2), (j1, j2))
    assert tens[0].shape == (1, i1, j1, n) and tens[1].shape == (n, i2, j2, 1)
    assert np.abs(O.mpo_contract(tens) - x).max() <= 1e-9
    # explicit sum for a few entries
    for (a1, a2, b1, b2) in [(0, 0, 0, 0), (i1 - 1, i2 - 1, j1 - 1, j2 - 1), (1, 5, 2, 3)]:
        want = sum(t_s[a1 * j1 + b1, r] * t_l[r, a2 * j2 + b2] for r in range(n))
        assert abs(want - x[a1 * i2 + a2, b1 * j2 + b2]) <= 1e-9


@pytest.mark.parametrize("fmt", [O.Format(4, 128, 128, 16, 8, 128, 1, 0, 2), O.Format(2, 64, 128, 8, 16, 256, 1, 0, 4),
                                 O.Format(8, 64, 64, 8, 8, 128, 1, 1, 2)])
def test_block_round_trip_within_the_half_step_bound(fmt):
    x = _block(5, fmt.block_tokens, fmt.head_dim, outliers=(2, 33))
    blk = O.compress_block(x, fmt)
    n = fmt.small_side
    assert blk.small.shape == (n, n) and blk.codes.shape == (fmt.block_tokens, fmt.head_dim)
    x_hat = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt)
    bound = O.reconstruction_bound(blk.small, blk.steps, fmt)
    t_l = O.token_major_to_large(blk.large32.astype(np.float64), fmt.j1, fmt.j2, fmt.i1)
    slack = O.unmatricise(2.0 ** -11 * np.abs(blk.small.astype(np.float64)) @ np.abs(t_l),
                          fmt.block_tokens, fmt.head_dim, fmt.i1, fmt.j1)
    err = np.abs(x_hat - x.astype(np.float64))
    assert (err <= bound + slack + 1e-9).all()
    if fmt.bits < 8:
        assert err.max() > 1e-3
        # the bond slices of a position swapped (rows a2*i1 + rho in another order) break it: the pin
        # sees the row layout
        perm = np.arange(fmt.block_tokens).reshape(-1, fmt.i1)[:, ::-1].reshape(-1)
        wrong = O.reconstruct_block(blk.small, blk.steps[perm], blk.codes[perm], fmt)
        assert not (np.abs(wrong - x.astype(np.float64)) <= bound + slack + 1e-9).all()


def _lossless_kv(seed, n_tok, d, qmax):
    r = np.random.default_rng(seed)
    c = r.integers(-qmax, qmax + 1, size=(n_tok, d))
    c[:, 0] = qmax
    c[:, d // 2] = -qmax
    step = 2.0 ** r.integers(-4, 1, size=(n_tok, 1))
    return (c * step).astype(np.float16)


@pytest.mark.parametrize("i1", [2, 4])
def test_attention_equals_dense_attention_when_the_code_is_lossless(i1):
    """T_S = I and exactly representable rows: the storage path with a token factor (row order
    a2*i1 + rho, small tensors of side i1*j1, masking by token index a1*i2 + a2) must reproduce
    brute-force dense attention on the original rows."""
    fmt = O.Format(4, 64, 128, 16, 8, 128, 1, 0, i1)
    bsz, hq, hkv, n_tok = 2, 4, 2, 300
    cache = O.empty_cache(fmt, bsz, hkv, 3)
    assert cache["k_small"].shape[-2:] == (16 * i1, 16 * i1)
    ks, vs = {}, {}
    for b in range(bsz):
        for h in range(hkv):
            ks[b, h] = _lossless_kv(10 * b + h, n_tok, 128, 7)
            vs[b, h] = _lossless_kv(100 + 10 * b + h, n_tok, 128, 7)
            O.compress_sequence(cache, fmt, b, h, ks[b, h], vs[b, h], identity_small=True)
    q = np.random.default_rng(5).standard_normal((bsz, hq, 128)).astype(np.float16)
    lens = np.array([300, 129], np.int32)
    out = O.attention_decode(cache, fmt, q, lens)
    for b in range(bsz):
        for i in range(hq):
            want = O.dense_attention(q[b, i], ks[b, i // 2][:lens[b]], vs[b, i // 2][:lens[b]])
            assert np.abs(out[b, i] - want).max() <= 1e-10


def test_token_factor_one_is_the_default_form_bit_for_bit():
    x = _block(7)
    a = O.compress_block(x, O.Format(4, 128, 128, 16, 8, 128))
    b = O.compress_block(x, O.Format(4, 128, 128, 16, 8, 128, 1, 0, 1))
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.steps.view(np.uint16), b.steps.view(np.uint16))
    assert np.array_equal(a.small.view(np.uint16), b.small.view(np.uint16))


def test_compression_ratio_counts_the_larger_small_tensor():
    f1, f2 = O.Format(4, 128, 128, 16, 8, 128), O.Format(4, 128, 128, 16, 8, 128, 1, 0, 2)
    assert O.cache_bytes_per_block(f2) - O.cache_bytes_per_block(f1) == (32 * 32 - 16 * 16) * 2
    assert abs(O.compression_ratio(f2) - (128 * 128 * 4 + 32 * 32 * 16 + 128 * 16) / (128 * 128 * 16.0)) < 1e-15


def test_format_rejects_shapes_without_a_full_bond():
    with pytest.raises(ValueError):
        O.Format(4, 128, 128, 16, 8, 128, 8, 0, 2).check()      # three tensors and a token factor
    with pytest.raises(ValueError):
        O.Format(4, 128, 128, 16, 8, 128, 1, 0, 3).check()      # 3 does not divide 128
