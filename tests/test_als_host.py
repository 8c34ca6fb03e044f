"""Host-side R x R algebra of the ALS update (no GPU): the library's pseudo-inverse against numpy's."""
import numpy as np
import pytest

from paper_1904_03329_amd import binding as B


@pytest.mark.parametrize("n", [1, 8, 32, 128])
def test_positive_definite_gram_products(n):
    rng = np.random.default_rng(n)
    a = rng.uniform(0, 1, (300, n))
    b = rng.uniform(-1, 1, (200, n))
    v = (a.T @ a) * (b.T @ b)
    got = B.sym_pinv(v)
    np.testing.assert_allclose(got, np.linalg.inv(v), rtol=1e-9, atol=1e-12 * np.abs(got).max())


@pytest.mark.parametrize("n", [4, 32])
def test_rank_deficient_products_take_the_pseudo_inverse(n):
    rng = np.random.default_rng(10 + n)
    a = rng.uniform(0, 1, (50, n))
    b = rng.uniform(0, 1, (60, n))
    a[:, 1] = a[:, 0]
    b[:, 1] = b[:, 0]              # two identical components: V has two equal rows
    v = (a.T @ a) * (b.T @ b)
    got = B.sym_pinv(v)
    want = np.linalg.pinv(v, hermitian=True)
    np.testing.assert_allclose(got, want, rtol=1e-7, atol=1e-9 * np.abs(want).max())
    # the four Moore-Penrose conditions, independent of numpy's routine
    np.testing.assert_allclose(v @ got @ v, v, atol=1e-9 * np.abs(v).max())
    np.testing.assert_allclose(got @ v @ got, got, atol=1e-9 * np.abs(got).max())
    np.testing.assert_allclose(v @ got, (v @ got).T, atol=1e-9)


def test_zero_matrix_and_bad_arguments():
    assert np.all(B.sym_pinv(np.zeros((5, 5))) == 0)
    with pytest.raises(B.HbcsfError):
        B.sym_pinv(np.zeros((129, 129)))
