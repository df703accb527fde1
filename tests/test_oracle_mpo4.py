"""Pins for the oracle's four-tensor form (Preliminary, Eq. 2 with n = 4; Section 4.3 "Analysis of
Length of Local Tensors"): factor shapes I = 1 * i2 * i3 * i4, J = j1 * j2 * 1 * 1, T_2 quantized,
T_3 [i3*i4, i3, i4] and T_4 [i4, i4] on the token side.  The HIP library has no such format; these
tests are the whole of its coverage."""
import numpy as np
import pytest

from oracle import decoquant_oracle as O


def _outlier_block(seed, n_tok=128, d=128, n_out=4, scale=20.0):
    r = np.random.default_rng(seed)
    x = r.standard_normal((n_tok, d)) * np.exp(0.5 * r.standard_normal((n_tok, 1)))
    x[:, r.choice(d, n_out, replace=False)] *= scale
    return x.astype(np.float16)


@pytest.mark.parametrize("n_tok,d,j1,i3,i4", [(128, 128, 16, 4, 4), (256, 64, 8, 4, 2), (32, 16, 4, 2, 2), (128, 128, 16, 2, 8)])
def test_four_tensors_reproduce_the_matrix_exactly(n_tok, d, j1, i3, i4):
    x = _outlier_block(7, n_tok, d, 2).astype(np.float64)
    t_1, t_2, t_3, t_4 = O.mpo4_split(x, j1, i3, i4)
    run = i3 * i4
    assert t_1.shape == (j1, j1) and t_2.shape == (j1, n_tok // run, d // j1, run)
    assert t_3.shape == (run, i3, i4) and t_4.shape == (i4, i4)
    rec = O.mpo4_contract(t_1, t_2, t_3, t_4)
    assert np.linalg.norm(rec - x) <= 1e-10 * np.linalg.norm(x)


def test_contraction_against_explicit_loops_on_a_tiny_case():
    # X[(a2, a3, a4), (b1, b2)] = sum_{r, e, f} T_1[b1, r] T_2[r, a2, b2, e] T_3[e, a3, f] T_4[f, a4], written out
    r = np.random.default_rng(3)
    j1, i2, j2, i3, i4 = 2, 2, 2, 2, 3
    run = i3 * i4
    t_1, t_2 = r.standard_normal((j1, j1)), r.standard_normal((j1, i2, j2, run))
    t_3, t_4 = r.standard_normal((run, i3, i4)), r.standard_normal((i4, i4))
    got = O.mpo4_contract(t_1, t_2, t_3, t_4)
    assert got.shape == (i2 * run, j1 * j2)
    for a2 in range(i2):
        for a3 in range(i3):
            for a4 in range(i4):
                for b1 in range(j1):
                    for b2 in range(j2):
                        want = sum(t_1[b1, rr] * t_2[rr, a2, b2, e] * t_3[e, a3, f] * t_4[f, a4]
                                   for rr in range(j1) for e in range(run) for f in range(i4))
                        assert abs(got[(a2 * i3 + a3) * i4 + a4, b1 * j2 + b2] - want) <= 1e-12


def test_gauge_and_agreement_with_the_general_decomposition():
    x = _outlier_block(11).astype(np.float64)
    t_1, t_2, t_3, t_4 = O.mpo4_split(x, 16, 4, 4)
    # first cut as in the two-tensor form
    sv = np.linalg.svd(O.matricise(x, 1, 16), compute_uv=False)
    assert np.allclose(np.linalg.norm(t_1, axis=0), sv, rtol=1e-10)
    # T_2 as a (r, a2, b2) x e matrix and T_3 as an (e, a3) x f matrix have orthonormal columns
    a = t_2.reshape(-1, 16)
    assert np.abs(a.T @ a - np.eye(16)).max() <= 1e-12
    b = t_3.reshape(-1, 4)
    assert np.abs(b.T @ b - np.eye(4)).max() <= 1e-12
    # so T_4 carries the last cut's singular values (orthogonal rows) and, the right factor of the first
    # cut having 16 orthonormal rows, their squares add up to 16
    gram = t_4 @ t_4.T
    assert np.abs(gram - np.diag(np.diag(gram))).max() <= 1e-12
    assert abs(np.trace(gram) - 16.0) <= 1e-10
    # same product as the general sequential-SVD decomposition with these factor shapes, and as the
    # two- and three-tensor forms
    general = O.mpo_contract(O.mpo_decompose(x, (1, 8, 4, 4), (16, 8, 1, 1)))
    mine = O.mpo4_contract(t_1, t_2, t_3, t_4)
    assert np.abs(general - mine).max() <= 1e-9
    assert np.abs(O.mpo3_contract(*O.mpo3_split(x, 16, 8)) - mine).max() <= 1e-9


def test_one_token_per_run_on_the_last_factor_is_the_three_tensor_form():
    # i4 = 1: the third cut splits off a 1 x 1 tensor, the norm of what the second cut left;
    # T_3 * T_4 is the three-tensor form's T_3 (up to the sign of each row), T_2 its T_2
    x = _outlier_block(4).astype(np.float64)
    t_1, t_2, t_3, t_4 = O.mpo4_split(x, 16, 8, 1)
    u_1, u_2, u_3 = O.mpo3_split(x, 16, 8)
    assert t_4.shape == (1, 1) and t_3.shape == (8, 8, 1)
    joined = t_3[:, :, 0] * t_4[0, 0]
    for e in range(8):
        s = 1.0 if np.abs(joined[e] - u_3[e]).max() <= np.abs(joined[e] + u_3[e]).max() else -1.0
        assert np.abs(s * joined[e] - u_3[e]).max() <= 1e-9
        assert np.abs(s * t_2[..., e] - u_2[..., e]).max() <= 1e-9
    assert np.abs(t_1 - u_1).max() <= 1e-12


def test_separable_token_structure_lands_in_the_first_rows():
    # X[(a2, a3, a4), c] = u[a3] * w[a4] * Y[a2, c]: both later cuts have rank one; T_4's only row
    # is sqrt(16) * w / |w| up to sign and T_3's only column (e = 0) is u / |u|
    r = np.random.default_rng(5)
    u, w = r.standard_normal(4), r.standard_normal(4)
    y = r.standard_normal((8, 128))
    x = (y[:, None, None, :] * u[None, :, None, None] * w[None, None, :, None]).reshape(128, 128)
    _, _, t_3, t_4 = O.mpo4_split(x, 16, 4, 4)
    assert np.abs(t_4[1:]).max() <= 1e-6
    want = 4.0 * w / np.linalg.norm(w)
    assert min(np.abs(t_4[0] - want).max(), np.abs(t_4[0] + want).max()) <= 1e-9
    col = t_3[0, :, 0]
    want = u / np.linalg.norm(u)
    assert min(np.abs(col - want).max(), np.abs(col + want).max()) <= 1e-9


@pytest.mark.parametrize("bits,group", [(4, 128), (2, 64), (8, 128)])
def test_reconstruction_error_within_the_half_step_bound(bits, group):
    fmt = O.Format(bits, group, 128, 16, 8, 128, 4, 0, 1, 4)
    x = _outlier_block(1)
    blk = O.compress_block(x, fmt)
    assert blk.small3.shape == (16, 4, 4) and blk.small4.shape == (4, 4) and blk.small4.dtype == np.float16
    x_hat = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt, blk.small3, blk.small4)
    bound = O.reconstruction_bound(blk.small, blk.steps, fmt, blk.small3, blk.small4)
    # plus the fp16 rounding of T_1, T_3 and T_4 (2^-11 relative each) and fp32 of T_2
    t_2 = np.abs(O.token_major_to_middle(blk.large32.astype(np.float64), 16, 8, 16))
    tok = np.einsum("def,fg->deg", np.abs(blk.small3.astype(np.float64)), np.abs(blk.small4.astype(np.float64))).reshape(16, 16)
    right = np.einsum("racd,de->raec", t_2, tok).reshape(16, 1024)
    slack = O.unmatricise(1.5 * 2.0 ** -10 * np.abs(blk.small.astype(np.float64)) @ right, 128, 128, 1, 16)
    err = np.abs(x_hat - x.astype(np.float64))
    assert (err <= bound + slack + 1e-9).all()
    if bits < 8:
        assert err.max() > 1e-3
    # The worst-case bound sums magnitudes over the 16 bond values e and is loose (an order of
    # magnitude above the error at 4 bits), so the index order of the token-side tensors is pinned by
    # what a swap does to the error itself, at 8 bits, where the code error is small: a transposed
    # T_4, or T_3 with its token and bond index swapped, is several times further from the block.
    if bits == 8:
        good = np.linalg.norm(x_hat - x.astype(np.float64))
        wrong = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt, blk.small3, blk.small4.T.copy())
        assert np.linalg.norm(wrong - x.astype(np.float64)) > 4.0 * good
        wrong = O.reconstruct_block(blk.small, blk.steps, blk.codes, fmt, blk.small3.transpose(0, 2, 1).copy(), blk.small4)
        assert np.linalg.norm(wrong - x.astype(np.float64)) > 4.0 * good


def test_attention_on_an_eight_bit_four_tensor_cache_is_close_to_dense_attention():
    # storage round trip (pack, T_3 and T_4 arrays, load) + decode; 8-bit codes leave ~1e-2 relative
    fmt = O.Format(8, 128, 128, 16, 8, 128, 4, 0, 1, 4)
    bsz, hq, hkv, n_tok = 2, 4, 2, 256
    cache = O.empty_cache(fmt, bsz, hkv, 2)
    assert cache["k_small3"].shape == (bsz, hkv, 2, 16, 16) and cache["v_small4"].shape == (bsz, hkv, 2, 4, 4)
    r = np.random.default_rng(6)
    ks, vs = {}, {}
    for b in range(bsz):
        for h in range(hkv):
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


def test_parameter_count_of_the_four_tensor_form():
    # Eq. 4 with the two extra small tensors: 16*4*4 + 4*4 more 16-bit parameters per block
    f2, f4 = O.Format(4, 128, 128, 16, 8, 128), O.Format(4, 128, 128, 16, 8, 128, 4, 0, 1, 4)
    extra = 16 * 4 * 4 + 4 * 4
    assert abs(O.compression_ratio(f4) - O.compression_ratio(f2) - extra * 16 / (128 * 128 * 16.0)) <= 1e-15
    assert O.cache_bytes_per_block(f4) == O.cache_bytes_per_block(f2) + 2 * extra
    with pytest.raises(ValueError):
        O.Format(4, 128, 128, 16, 8, 128, 1, 0, 1, 4).check()      # four tensors need i3 > 1
    with pytest.raises(ValueError):
        O.Format(4, 128, 128, 16, 8, 128, 8, 0, 1, 32).check()     # i3 * i4 must divide the block
