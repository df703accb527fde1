"""Pins for the oracle's three-tensor form (Preliminary, Eq. 2 with n = 3; Section 4.3 "Analysis of
Length of Local Tensors"): factor shapes I = 1 * (T_b / i3) * i3, J = j1 * j2 * 1, middle tensor
quantized, the third tensor i3 x i3 on the token side."""
import numpy as np
import pytest

from oracle import decoquant_oracle as O


def _outlier_block(seed, n_tok=128, d=128, n_out=4, scale=20.0):
    r = np.random.default_rng(seed)
    x = r.standard_normal((n_tok, d)) * np.exp(0.5 * r.standard_normal((n_tok, 1)))
    x[:, r.choice(d, n_out, replace=False)] *= scale
    return x.astype(np.float16)


@pytest.mark.parametrize("n_tok,d,j1,i3", [(128, 128, 16, 8), (256, 64, 8, 8), (32, 16, 4, 4), (128, 128, 16, 2)])
def test_three_tensors_reproduce_the_matrix_exactly(n_tok, d, j1, i3):
    x = _outlier_block(7, n_tok, d, 2).astype(np.float64)
    t_1, t_2, t_3 = O.mpo3_split(x, j1, i3)
    assert t_1.shape == (j1, j1) and t_2.shape == (j1, n_tok // i3, d // j1, i3) and t_3.shape == (i3, i3)
    rec = O.mpo3_contract(t_1, t_2, t_3)
    assert np.linalg.norm(rec - x) <= 1e-10 * np.linalg.norm(x)


def test_contraction_against_explicit_loops_on_a_tiny_case():
    # X[(a2, a3), (b1, b2)] = sum_r sum_e T_1[b1, r] T_2[r, a2, b2, e] T_3[e, a3], written out
    r = np.random.default_rng(3)
    j1, i2, j2, i3 = 2, 3, 2, 2
    t_1, t_2, t_3 = r.standard_normal((j1, j1)), r.standard_normal((j1, i2, j2, i3)), r.standard_normal((i3, i3))
    got = O.mpo3_contract(t_1, t_2, t_3)
    for a2 in range(i2):
        for a3 in range(i3):
            for b1 in range(j1):
                for b2 in range(j2):
                    want = sum(t_1[b1, rr] * t_2[rr, a2, b2, e] * t_3[e, a3] for rr in range(j1) for e in range(i3))
                    assert abs(got[a2 * i3 + a3, b1 * j2 + b2] - want) <= 1e-12


def test_gauge_singular_values_stay_in_the_small_tensors():
    x = _outlier_block(11).astype(np.float64)
    t_1, t_2, t_3 = O.mpo3_split(x, 16, 8)
    # first cut: the columns of T_1 carry the singular values of the regrouped block
    sv = np.linalg.svd(O.matricise(x, 1, 16), compute_uv=False)
    assert np.allclose(np.linalg.norm(t_1, axis=0), sv, rtol=1e-10)
    # the middle tensor has orthonormal columns as a (r, a2, b2) x e matrix ...
    a = t_2.reshape(-1, 8)
    assert np.abs(a.T @ a - np.eye(8)).max() <= 1e-12
    # ... so T_3 carries the second cut's singular values: orthogonal rows, and since the right
    # factor of the first cut has 16 orthonormal rows, their squares add up to 16
    gram = t_3 @ t_3.T
    assert np.abs(gram - np.diag(np.diag(gram))).max() <= 1e-12
    assert abs(np.trace(gram) - 16.0) <= 1e-10
    # same product as the general sequential-SVD decomposition with these factor shapes
    general = O.mpo_contract(O.mpo_decompose(x, (1, 16, 8), (16, 8, 1)))
    assert np.abs(general - O.mpo3_contract(t_1, t_2, t_3)).max() <= 1e-9


def test_rank_one_token_structure_lands_in_one_row_of_the_third_tensor():
    # X[(a2, a3), c] = w[a3] * Y[a2, c]: the second cut has rank one and T_3's only row is
    # sqrt(16) * w / |w| up to sign (the right factor of the first cut has squared norm 16)
    r = np.random.default_rng(5)
    w = r.standard_normal(8)
    y = r.standard_normal((16, 128))
    x = (y[:, None, :] * w[None, :, None]).reshape(128, 128)
    _, _, t_3 = O.mpo3_split(x, 16, 8)
    assert np.abs(t_3[1:]).max() <= 1e-7
    want = 4.0 * w / np.linalg.norm(w)
    assert min(np.abs(t_3[0] - want).max(), np.abs(t_3[0] + want).max()) <= 1e-9


def test_middle_tensor_row_layout():
    r = np.random.default_rng(2)
    t_2 = r.standard_normal((4, 3, 2, 2)).astype(np.float32).astype(np.float64)   # r, a2, b2, e
    kp = O.middle_to_token_major(t_2)
    assert kp.shape == (6, 8) and kp.dtype == np.float32
    for rr in range(4):
        for a2 in range(3):
            for b2 in range(2):
                for e in range(2):
                    assert kp[a2 * 2 + e, rr * 2 + b2] == t_2[rr, a2, b2, e]
    assert np.array_equal(O.token_major_to_middle(kp.astype(np.float64), 4, 2, 2), t_2)


@pytest.mark.parametrize("bits,group", [(4, 128), (2, 64), (8, 128)])
def test_reconstruction_error_within_the_half_step_bound(bits, group):
    fmt = O.Format(bits, group, 128, 16, 8, 128, 8)
    x = _outlier_block(1)
    blk = O.compress_block(x, fmt)
    assert blk.small3.shape == (8, 8) and blk.small3.dtype == np.float16
    x_hat = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt, blk.small3)
    bound = O.reconstruction_bound(blk.small, blk.steps, fmt, blk.small3)
    # plus the fp16 rounding of T_1 and T_3 (2^-11 relative each) and fp32 of T_2
    t_2 = np.abs(O.token_major_to_middle(blk.large32.astype(np.float64), 16, 8, 8))
    right = np.einsum("racd,de->raec", t_2, np.abs(blk.small3.astype(np.float64))).reshape(16, 1024)
    slack = O.unmatricise(2.0 ** -10 * np.abs(blk.small.astype(np.float64)) @ right, 128, 128, 1, 16)
    err = np.abs(x_hat - x.astype(np.float64))
    assert (err <= bound + slack + 1e-9).all()
    if bits < 8:
        assert err.max() > 1e-3
    # a transposed third tensor breaks it: the pin is sensitive to its index order
    wrong = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt, blk.small3.T.copy())
    assert not (np.abs(wrong - x.astype(np.float64)) <= bound + slack + 1e-9).all()


def test_attention_on_an_eight_bit_three_tensor_cache_is_close_to_dense_attention():
    # storage round trip (pack, both T_3 layouts, load) + decode; 8-bit codes leave ~1e-2 relative
    fmt = O.Format(8, 128, 128, 16, 8, 128, 8)
    bsz, hq, hkv, n_tok = 2, 4, 2, 256
    cache = O.empty_cache(fmt, bsz, hkv, 2)
    assert cache["k_small3"].shape == (bsz, hkv, 2, 8, 8)
    r = np.random.default_rng(6)
    ks, vs = {}, {}
    for b in range(bsz):
        for h in range(hkv):
            # no outlier channels here: with them the softmax is so peaked that an 8-bit code moves
            # the output by several percent (in the two-tensor form as well)
            ks[b, h] = _outlier_block(10 * b + h, n_tok, scale=1.0)
            vs[b, h] = _outlier_block(100 + 10 * b + h, n_tok, scale=1.0)
            O.compress_sequence(cache, fmt, b, h, ks[b, h], vs[b, h])
    q = r.standard_normal((bsz, hq, 128)).astype(np.float16)
    lens = np.array([256, 131], np.int32)
    out = O.attention_decode(cache, fmt, q, lens)
    for b in range(bsz):
        for i in range(hq):
            h = i // 2
            want = O.dense_attention(q[b, i], ks[b, h][:lens[b]], vs[b, h][:lens[b]])
            assert np.abs(out[b, i] - want).max() <= 0.02 * np.abs(want).max() + 0.01


def test_two_and_three_tensor_forms_agree_when_nothing_is_quantized():
    x = _outlier_block(9).astype(np.float64)
    t_s, t_l = O.mpo_split(x, 16)
    t_1, t_2, t_3 = O.mpo3_split(x, 16, 8)
    two = O.unmatricise(t_s @ t_l, 128, 128, 1, 16)
    assert np.abs(two - O.mpo3_contract(t_1, t_2, t_3)).max() <= 1e-9
    # Eq. 4 with the extra small tensor: 64 more 16-bit parameters per block
    f2, f3 = O.Format(4, 128, 128, 16, 8, 128), O.Format(4, 128, 128, 16, 8, 128, 8)
    assert abs(O.compression_ratio(f3) - O.compression_ratio(f2) - 64 * 16 / (128 * 128 * 16.0)) <= 1e-15
    assert O.cache_bytes_per_block(f3) == O.cache_bytes_per_block(f2) + 128
