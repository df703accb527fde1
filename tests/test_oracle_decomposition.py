"""Pins for the oracle's MPO decomposition (Preliminary Eq. 2; Section 3.1 Eq. 3)."""
import numpy as np
import pytest

from oracle import decoquant_oracle as O


def _block(seed, n_tok=128, d=128, outliers=(3, 40, 77, 100), scale=20.0):
    r = np.random.default_rng(seed)
    x = r.standard_normal((n_tok, d))
    x[:, list(outliers)] *= scale
    return x.astype(np.float16).astype(np.float64)


def test_matricise_matches_index_formula():
    # Eq. 2 with n = 2: M[(a1,b1),(a2,b2)] = X[a1*i2+a2, b1*j2+b2], checked by explicit loops.
    i1, i2, j1, j2 = 2, 3, 4, 5
    x = np.arange(i1 * i2 * j1 * j2, dtype=np.float64).reshape(i1 * i2, j1 * j2)
    m = O.matricise(x, i1, j1)
    assert m.shape == (i1 * j1, i2 * j2)
    for a1 in range(i1):
        for b1 in range(j1):
            for a2 in range(i2):
                for b2 in range(j2):
                    assert m[a1 * j1 + b1, a2 * j2 + b2] == x[a1 * i2 + a2, b1 * j2 + b2]
    assert np.array_equal(O.unmatricise(m, i1 * i2, j1 * j2, i1, j1), x)


@pytest.mark.parametrize("sigma_in", ["small", "large"])
@pytest.mark.parametrize("shape", [(128, 128, 16), (256, 64, 8), (128, 128, 32)])
def test_split_is_exact(sigma_in, shape):
    n_tok, d, j1 = shape
    x = _block(1, n_tok, d, outliers=(1, 9))
    t_s, t_l = O.mpo_split(x, j1, 1, sigma_in)
    m = O.matricise(x, 1, j1)
    assert t_s.shape == (j1, j1) and t_l.shape == (j1, n_tok * d // j1)
    rel = np.linalg.norm(t_s @ t_l - m) / np.linalg.norm(m)
    assert rel <= 1e-10
    # the local tensors hold a few more parameters than the matrix (Section 3.3): exactly j1^2 more
    assert t_s.size + t_l.size == x.size + j1 * j1
    if sigma_in == "small":
        assert np.abs(t_l @ t_l.T - np.eye(j1)).max() <= 1e-12
    else:
        assert np.abs(t_s.T @ t_s - np.eye(j1)).max() <= 1e-12


def test_split_small_share_is_in_the_papers_regime():
    # Section 3.1 quotes T_S at 0.6 % of the parameters; the default shapes give 0.2-1.5 %.
    for tb in (128, 256, 1024):
        share = 16 * 16 / (16 * 16 + 16 * tb * 8)
        assert 0.001 < share < 0.02


def test_split_j1_equal_one_is_a_norm_and_a_direction():
    x = _block(2, 128, 64, outliers=(3, 40))
    t_s, t_l = O.mpo_split(x, 1)
    assert t_s.shape == (1, 1)
    assert abs(abs(t_s[0, 0]) - np.linalg.norm(x)) <= 1e-9
    assert np.allclose(t_s[0, 0] * t_l.reshape(128, 64), x, atol=1e-10)


def test_split_j2_equal_one_is_the_textbook_svd_of_the_transpose():
    x = _block(3, 128, 16, outliers=(5,))
    t_s, t_l = O.mpo_split(x, 16)          # M = X^T  (16 x 128)
    assert np.allclose(t_s @ t_l, x.T, atol=1e-10)
    sv = np.linalg.svd(x, compute_uv=False)
    assert np.allclose(np.linalg.norm(t_s, axis=0), sv, rtol=1e-12)
    # columns of T_S are orthogonal (they are U * sigma)
    g = t_s.T @ t_s
    assert np.abs(g - np.diag(np.diag(g))).max() <= 1e-9 * g.max()


def test_split_sign_convention():
    x = _block(4)
    _, t_l = O.mpo_split(x, 16)
    piv = np.abs(t_l).argmax(axis=1)
    assert (t_l[np.arange(16), piv] > 0).all()


def test_zero_rows_do_not_break_exactness():
    x = _block(5)
    x[37:] = 0.0                       # partially filled block
    t_s, t_l = O.mpo_split(x, 16)
    assert np.linalg.norm(t_s @ t_l - O.matricise(x, 1, 16)) <= 1e-10 * np.linalg.norm(x)
    x[1:] = 0.0                        # rank-deficient: 8 non-zero columns < 16 rows
    t_s, t_l = O.mpo_split(x, 16)
    assert np.linalg.norm(t_s @ t_l - O.matricise(x, 1, 16)) <= 1e-10 * np.linalg.norm(x)


@pytest.mark.parametrize("ishape,jshape", [((1, 32), (8, 4)), ((2, 16), (4, 8)),
                                           ((2, 4, 4), (2, 2, 8)), ((1, 2, 2, 8), (2, 2, 2, 4))])
def test_general_mpo_contracts_back(ishape, jshape):
    r = np.random.default_rng(6)
    w = r.standard_normal((int(np.prod(ishape)), int(np.prod(jshape))))
    ts = O.mpo_decompose(w, ishape, jshape)
    assert len(ts) == len(ishape)
    d_prev = 1
    for k, t in enumerate(ts):
        assert t.shape[0] == d_prev and t.shape[1] == ishape[k] and t.shape[2] == jshape[k]
        d_prev = t.shape[3]
    assert d_prev == 1
    assert np.abs(O.mpo_contract(ts) - w).max() <= 1e-10


def test_two_site_split_is_an_mpo_in_the_sense_of_eq2():
    x = _block(7, 128, 64, outliers=(2, 50))
    t_s, t_l = O.mpo_split(x, 8)
    ts = O.as_local_tensors(t_s, t_l, 1, 8, 128, 8)
    assert ts[0].shape == (1, 1, 8, 8) and ts[1].shape == (8, 128, 8, 1)
    assert np.abs(O.mpo_contract(ts) - x).max() <= 1e-9


def test_large_tensor_is_narrower_than_the_matrix():
    # Section 3.1 / Appendix A.1: the interquartile range of T_L is far below the matrix's.
    def iqr(a):
        q1, q3 = np.percentile(a, [25, 75])
        return q3 - q1
    for seed in range(3):
        x = _block(10 + seed)
        t_s, t_l = O.mpo_split(x, 16)
        assert iqr(t_l) < 0.2 * iqr(x)
        assert np.abs(t_l).max() <= 1.0 + 1e-12     # orthonormal rows bound every entry by 1
