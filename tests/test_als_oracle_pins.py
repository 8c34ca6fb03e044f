"""Pins of the CPD-ALS oracle (no GPU): textbook least squares per mode update, the exact-model fixed point,
monotone residual, and agreement of its MTTKRP with the C oracle."""
import numpy as np

from oracle import cpd_als


def _dense_model(factors, lam):
    rank = len(lam)
    x = 0
    for r in range(rank):
        t = lam[r]
        for f in factors:
            t = np.multiply.outer(t, f[:, r])
        x = x + t
    return x


def _coo_of_dense(x):
    grid = np.meshgrid(*[np.arange(d) for d in x.shape], indexing="ij")
    return [g.ravel().astype(np.uint32) for g in grid], x.ravel()


def _khatri_rao_all_but(factors, n):
    rank = factors[0].shape[1]
    kr = np.ones((1, rank))
    for m, a in enumerate(factors):
        if m != n:
            kr = (a[:, None, :] * kr[None, :, :]).reshape(-1, rank)
    return kr


def test_each_mode_update_is_the_least_squares_solution():
    """Eq. 2: A_n minimises || X_(n) - A (Khatri-Rao)^T ||_F; compare with numpy.linalg.lstsq on the explicit
    system.  Only the first update of an iteration sees the input factors, so check mode by mode."""
    rng = np.random.default_rng(1)
    dims = (6, 5, 4)
    x = rng.normal(size=dims)
    inds, vals = _coo_of_dense(x)
    for n in range(3):
        facs = [rng.uniform(0.1, 1, size=(d, 3)) for d in dims]
        m_n = cpd_als.mttkrp(dims, inds, vals, facs, n)
        v = np.ones((3, 3))
        for m in range(3):
            if m != n:
                v *= facs[m].T @ facs[m]
        got = m_n @ np.linalg.pinv(v)
        kr = _khatri_rao_all_but(facs, n)
        xn = np.reshape(np.moveaxis(x, n, 0), (dims[n], -1), order="F")
        want = np.linalg.lstsq(kr, xn.T, rcond=None)[0].T
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)


def test_exact_low_rank_tensor_is_a_fixed_point():
    rng = np.random.default_rng(2)
    dims = (7, 6, 5, 4)
    rank = 3
    facs = [rng.uniform(0.2, 1, size=(d, rank)) for d in dims]
    facs = [f / np.linalg.norm(f, axis=0) for f in facs]
    lam = np.array([3.0, 2.0, 0.5])
    x = _dense_model(facs, lam)
    inds, vals = _coo_of_dense(x)
    start = [f.copy() for f in facs]
    start[0] = start[0] * lam            # unnormalised model of the same tensor
    new, new_lam = cpd_als.als_iteration(dims, inds, vals, start)
    for f, g in zip(facs, new):
        np.testing.assert_allclose(g, f, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(new_lam, lam, rtol=1e-8)
    np.testing.assert_allclose(cpd_als.model_values(inds, new, new_lam), vals, rtol=1e-8, atol=1e-10)


def test_residual_never_increases():
    rng = np.random.default_rng(3)
    dims = (8, 7, 6)
    x = rng.normal(size=dims) * (rng.uniform(size=dims) < 0.3)
    inds, vals = _coo_of_dense(x)
    facs = [rng.uniform(0, 1, size=(d, 4)) for d in dims]
    lam = np.ones(4)
    prev = np.inf
    for _ in range(6):
        facs, lam = cpd_als.als_iteration(dims, inds, vals, [f * (lam if i == 0 else 1) for i, f in enumerate(facs)])
        res = np.linalg.norm(_dense_model(facs, lam) - x)
        assert res <= prev * (1 + 1e-12)
        prev = res
    for f in facs:
        np.testing.assert_allclose(np.linalg.norm(f, axis=0), 1.0, rtol=1e-12)


def test_its_mttkrp_agrees_with_the_c_oracle(oracle):
    rng = np.random.default_rng(4)
    dims = (30, 20, 10, 5)
    n = 2000
    inds = [rng.integers(0, d, n).astype(np.uint32) for d in dims]
    vals = rng.uniform(-1, 1, n).astype(np.float32)
    facs = [rng.uniform(0, 1, size=(d, 8)).astype(np.float32) for d in dims]
    for mode in range(4):
        np.testing.assert_allclose(cpd_als.mttkrp(dims, inds, vals, facs, mode),
                                   oracle.mttkrp(dims, inds, vals, facs, mode), rtol=1e-12, atol=1e-13)


def test_fit_equals_the_dense_residual():
    rng = np.random.default_rng(5)
    dims = (6, 5, 4)
    x = rng.normal(size=dims) * (rng.uniform(size=dims) < 0.4)
    nz = np.nonzero(x)
    inds = [i.astype(np.uint32) for i in nz]
    vals = x[nz]
    facs = [rng.uniform(0, 1, size=(d, 3)) for d in dims]
    lam = rng.uniform(0.5, 2, size=3)
    want = 1.0 - np.linalg.norm(_dense_model(facs, lam) - x) / np.linalg.norm(x)
    np.testing.assert_allclose(cpd_als.fit(dims, inds, vals, facs, lam), want, rtol=1e-10)


def test_planted_mistakes_fail_the_least_squares_pin():
    """The pin has teeth: plausible wrong updates (the updated mode's own Gram matrix in the Hadamard product, an
    element-wise reciprocal instead of the pseudo-inverse, the MTTKRP of another mode) do not solve Eq. 2."""
    rng = np.random.default_rng(6)
    dims = (6, 5, 4)
    x = rng.normal(size=dims)
    inds, vals = _coo_of_dense(x)
    facs = [rng.uniform(0.1, 1, size=(d, 3)) for d in dims]
    n = 1
    kr = _khatri_rao_all_but(facs, n)
    xn = np.reshape(np.moveaxis(x, n, 0), (dims[n], -1), order="F")
    want = np.linalg.lstsq(kr, xn.T, rcond=None)[0].T
    m_n = cpd_als.mttkrp(dims, inds, vals, facs, n)
    v = (facs[0].T @ facs[0]) * (facs[2].T @ facs[2])
    np.testing.assert_allclose(m_n @ np.linalg.pinv(v), want, rtol=1e-9, atol=1e-10)       # the correct update
    wrong = [
        m_n @ np.linalg.pinv(v * (facs[1].T @ facs[1])),
        m_n @ (1.0 / v),
        m_n @ np.linalg.pinv((facs[0].T @ facs[0]) @ (facs[2].T @ facs[2])),               # matrix, not Hadamard, product
    ]
    for w in wrong:
        assert np.max(np.abs(w - want)) > 1e-3 * np.max(np.abs(want))


def test_gram_is_the_sum_of_row_outer_products():
    """The Gram matrix of Eq. 3 written out entry by entry: S[r][s] = sum_i A[i][r] A[i][s]."""
    rng = np.random.default_rng(77)
    a = rng.uniform(-1, 1, size=(37, 5)).astype(np.float32)
    want = np.zeros((5, 5))
    for i in range(37):
        for r in range(5):
            for s in range(5):
                want[r, s] += float(a[i, r]) * float(a[i, s])
    got = cpd_als.gram(a)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(np.diag(got), (a.astype(np.float64) ** 2).sum(axis=0), rtol=1e-13)
    assert np.array_equal(got, got.T)
    assert np.array_equal(cpd_als.gram(np.zeros((0, 4), np.float32)), np.zeros((4, 4)))
