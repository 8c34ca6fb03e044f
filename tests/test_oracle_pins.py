"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test fixes the oracle to the mathematics of Section II-C: the matricised tensor times an
explicit Khatri-Rao product (Eq. 4), the per-nonzero Hadamard form with its unfolding column
y = j + k*J (Eq. 5), closed forms, invariants, and textbook special cases computed by numpy /
scipy routines.  The paper prints no MTTKRP output values, so there is no numeric fixture of the
paper's own to compare with.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp


def _random_coo(rng, dims, nnz, unique=True):
    total = int(np.prod(dims))
    if unique:
        lin = rng.choice(total, size=min(nnz, total), replace=False)
    else:
        lin = rng.integers(0, total, size=nnz)
    inds = np.unravel_index(lin, dims)
    inds = [np.asarray(x, dtype=np.uint32) for x in inds]
    vals = rng.uniform(-1, 1, size=lin.shape[0]).astype(np.float32)
    return inds, vals


def _factors(rng, dims, rank):
    return [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]


def _dense(dims, inds, vals):
    x = np.zeros(dims, dtype=np.float64)
    np.add.at(x, tuple(i.astype(np.int64) for i in inds), vals.astype(np.float64))
    return x


def _unfold(x, n):
    """Mode-n matricisation, the first remaining mode varying fastest along the columns."""
    return np.reshape(np.moveaxis(x, n, 0), (x.shape[n], -1), order="F")


def _khatri_rao_all_but(factors, n):
    """Explicit Khatri-Rao product of all factors but the n-th, rows ordered like _unfold's columns."""
    rank = factors[0].shape[1] if n != 0 else factors[1].shape[1]
    kr = np.ones((1, rank), dtype=np.float64)
    for m, a in enumerate(factors):
        if m == n:
            continue
        a = a.astype(np.float64)
        kr = (a[:, None, :] * kr[None, :, :]).reshape(-1, rank)
    return kr


@pytest.mark.parametrize("dims", [(5, 4, 3), (2, 7, 3), (3, 4, 2, 5), (6, 1, 4), (2, 3, 4, 2, 3)])
@pytest.mark.parametrize("rank", [1, 3, 8])
def test_dense_matricised_times_khatri_rao(oracle, dims, rank):
    rng = np.random.default_rng(hash((dims, rank)) % 2**32)
    inds, vals = _random_coo(rng, dims, max(1, int(0.4 * np.prod(dims))))
    facs = _factors(rng, dims, rank)
    x = _dense(dims, inds, vals)
    for n in range(len(dims)):
        want = _unfold(x, n) @ _khatri_rao_all_but(facs, n)
        got = oracle.mttkrp(dims, inds, vals, facs, n)
        assert got.shape == (dims[n], rank)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_per_nonzero_hadamard_form_eq5(oracle):
    """Eq. 5 as printed for mode 1 of a 3-order tensor: column y pairs B(y % J) with C(y // J)."""
    rng = np.random.default_rng(5)
    dims = (4, 5, 3)
    I, J, K = dims
    inds, vals = _random_coo(rng, dims, 30)
    A, B, C = _factors(rng, dims, 4)
    x1 = _unfold(_dense(dims, inds, vals), 0)
    want = np.zeros((I, 4))
    for i in range(I):
        for y in range(J * K):
            want[i] += x1[i, y] * B[y % J].astype(np.float64) * C[y // J].astype(np.float64)
    np.testing.assert_allclose(oracle.mttkrp(dims, inds, vals, [A, B, C], 0), want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("order", [3, 4])
def test_rank_one_tensor_closed_form(oracle, order):
    """X = a o b o c (o d), all entries stored: M(i,r) = a_i * prod_m (x_m . A_m[:,r])."""
    rng = np.random.default_rng(order)
    dims = (4, 3, 5, 2)[:order]
    vecs = [rng.uniform(-1, 1, size=d).astype(np.float32) for d in dims]
    grid = np.meshgrid(*[np.arange(d) for d in dims], indexing="ij")
    inds = [g.ravel().astype(np.uint32) for g in grid]
    dense = vecs[0].astype(np.float64)
    for v in vecs[1:]:
        dense = np.multiply.outer(dense, v.astype(np.float64))
    vals = dense.ravel().astype(np.float32)
    # The closed form must use the values as stored (rounded to fp32), so rebuild them from
    # exactly representable vectors: small dyadic rationals.
    vecs = [np.round(v * 8) / 8 for v in vecs]
    dense = vecs[0].astype(np.float64)
    for v in vecs[1:]:
        dense = np.multiply.outer(dense, v.astype(np.float64))
    vals = dense.ravel().astype(np.float32)
    assert np.array_equal(vals.astype(np.float64), dense.ravel())
    rank = 6
    facs = _factors(rng, dims, rank)
    for n in range(order):
        want = np.ones((dims[n], rank))
        want *= vecs[n][:, None]
        for m in range(order):
            if m != n:
                want *= (vecs[m].astype(np.float64) @ facs[m].astype(np.float64))[None, :]
        np.testing.assert_allclose(oracle.mttkrp(dims, inds, vals, facs, n), want, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("dims", [(30, 20, 10), (9, 8, 7, 6)])
def test_cross_mode_invariant(oracle, dims):
    """sum_{i,r} M^(n)(i,r) A_n(i,r) = sum_z v_z sum_r prod_m A_m(i_m,r), the same for every n."""
    rng = np.random.default_rng(len(dims))
    inds, vals = _random_coo(rng, dims, 500)
    facs = _factors(rng, dims, 5)
    direct = 0.0
    for z in range(vals.shape[0]):
        p = np.full(5, float(vals[z]))
        for m in range(len(dims)):
            p = p * facs[m][inds[m][z]].astype(np.float64)
        direct += p.sum()
    for n in range(len(dims)):
        s = float((oracle.mttkrp(dims, inds, vals, facs, n) * facs[n].astype(np.float64)).sum())
        assert abs(s - direct) <= 1e-11 * max(1.0, abs(direct))


def test_nonzero_order_and_partition_invariance(oracle):
    rng = np.random.default_rng(7)
    dims = (12, 9, 11)
    inds, vals = _random_coo(rng, dims, 400)
    facs = _factors(rng, dims, 8)
    perm = rng.permutation(vals.shape[0])
    parts = np.array_split(rng.permutation(vals.shape[0]), 5)
    for n in range(3):
        base = oracle.mttkrp(dims, inds, vals, facs, n)
        shuf = oracle.mttkrp(dims, [x[perm] for x in inds], vals[perm], facs, n)
        np.testing.assert_allclose(shuf, base, rtol=1e-12, atol=1e-13)
        total = sum(oracle.mttkrp(dims, [x[p] for x in inds], vals[p], facs, n) for p in parts)
        np.testing.assert_allclose(total, base, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(oracle.mttkrp(dims, inds, (-2 * vals).astype(np.float32), facs, n),
                                   -2 * base, rtol=1e-12, atol=1e-13)


def test_sparse_matrix_special_case_against_scipy(oracle):
    """K = 1 and C = 1: mode-1 MTTKRP is the sparse matrix product X(IxJ) @ B; mode 2 is X^T @ A."""
    rng = np.random.default_rng(11)
    I, J, R = 40, 33, 7
    inds, vals = _random_coo(rng, (I, J, 1), 300)
    A, B, _ = _factors(rng, (I, J, 1), R)
    C = np.ones((1, R), dtype=np.float32)
    x = sp.csr_matrix((vals.astype(np.float64), (inds[0].astype(np.int64), inds[1].astype(np.int64))), shape=(I, J))
    np.testing.assert_allclose(oracle.mttkrp((I, J, 1), inds, vals, [A, B, C], 0), x @ B.astype(np.float64),
                               rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.mttkrp((I, J, 1), inds, vals, [A, B, C], 1), x.T @ A.astype(np.float64),
                               rtol=1e-12, atol=1e-13)


def test_all_ones_rank_one_is_slice_sum(oracle):
    rng = np.random.default_rng(13)
    dims = (25, 6, 9, 4)
    inds, vals = _random_coo(rng, dims, 600)
    ones = [np.ones((d, 1), dtype=np.float32) for d in dims]
    for n in range(4):
        want = np.bincount(inds[n].astype(np.int64), weights=vals.astype(np.float64), minlength=dims[n])
        np.testing.assert_allclose(oracle.mttkrp(dims, inds, vals, ones, n)[:, 0], want, rtol=1e-12, atol=1e-13)


def test_single_nonzero_and_duplicates(oracle):
    rng = np.random.default_rng(17)
    dims = (3, 4, 5)
    A, B, C = _factors(rng, dims, 4)
    inds = [np.array([2], np.uint32), np.array([1], np.uint32), np.array([3], np.uint32)]
    vals = np.array([0.75], np.float32)
    got = oracle.mttkrp(dims, inds, vals, [A, B, C], 0)
    want = np.zeros((3, 4))
    want[2] = 0.75 * B[1].astype(np.float64) * C[3].astype(np.float64)
    np.testing.assert_array_equal(got, want)
    got = oracle.mttkrp(dims, inds, vals, [A, B, C], 2)
    want = np.zeros((5, 4))
    want[3] = 0.75 * A[2].astype(np.float64) * B[1].astype(np.float64)
    np.testing.assert_array_equal(got, want)
    # duplicate coordinates are separate nonzeros and add up
    inds2 = [np.repeat(x, 3) for x in inds]
    vals2 = np.array([0.75, 0.25, -0.5], np.float32)
    got = oracle.mttkrp(dims, inds2, vals2, [A, B, C], 0)
    np.testing.assert_allclose(got[2], 0.5 * B[1].astype(np.float64) * C[3].astype(np.float64), rtol=1e-15)


def test_planted_mistakes_are_caught(oracle):
    """The dense check must reject the plausible wrong formulas (swapped factors, dropped value,
    wrong target mode), i.e. the pins above are sharp enough to tell them apart."""
    rng = np.random.default_rng(19)
    dims = (4, 5, 6)
    inds, vals = _random_coo(rng, dims, 60)
    facs = _factors(rng, dims, 3)
    x = _dense(dims, inds, vals)
    good = _unfold(x, 0) @ _khatri_rao_all_but(facs, 0)
    got = oracle.mttkrp(dims, inds, vals, facs, 0)
    np.testing.assert_allclose(got, good, rtol=1e-12)
    # transposed pairing of the Khatri-Rao rows with the unfolding columns
    kr_swapped = (facs[1].astype(np.float64)[:, None, :] * facs[2].astype(np.float64)[None, :, :]).reshape(-1, 3)
    assert not np.allclose(_unfold(x, 0) @ kr_swapped, got, rtol=1e-6)
    # value dropped
    assert not np.allclose(oracle.mttkrp(dims, inds, np.ones_like(vals), facs, 0), got, rtol=1e-6)


def test_rows_variant_and_errors(oracle):
    rng = np.random.default_rng(23)
    dims = (50, 7, 8)
    inds, vals = _random_coo(rng, dims, 700)
    facs = _factors(rng, dims, 8)
    full = oracle.mttkrp(dims, inds, vals, facs, 0)
    rows = np.array([49, 0, 17, 3])
    np.testing.assert_array_equal(oracle.mttkrp_rows(dims, inds, vals, facs, 0, rows), full[rows])
    bad = [x.copy() for x in inds]
    bad[1][5] = 7
    with pytest.raises(RuntimeError):
        oracle.mttkrp(dims, bad, vals, facs, 0)


def test_workload_cfg1(oracle, synth):
    """The smallest benchmark configuration: 10,000 distinct uniform coordinates, R = 8."""
    t, facs, rank = synth.workload("cfg1")
    assert t.nnz == 10_000 and rank == 8 and t.dims == (100, 80, 60)
    keys = (t.inds[0].astype(np.int64) * 80 + t.inds[1]) * 60 + t.inds[2]
    assert np.unique(keys).shape[0] == t.nnz
    x = _dense(t.dims, t.inds, t.vals)
    for n in range(3):
        want = _unfold(x, n) @ _khatri_rao_all_but(facs, n)
        np.testing.assert_allclose(oracle.mttkrp(t.dims, t.inds, t.vals, facs, n), want, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("dims", [(60, 40, 30), (30, 12, 9, 7)])
def test_all_cores_variant_equals_the_oracle(oracle, dims):
    """The all-cores timing variant (atomic fp64 adds) is the same sum in another order: equal to the
    single-thread oracle within fp64 rounding, and against the dense definition (Eq. 4) directly."""
    rng = np.random.default_rng(41 + len(dims))
    inds, vals = _random_coo(rng, dims, 5000)
    facs = _factors(rng, dims, 8)
    x = _dense(dims, inds, vals)
    for n in range(len(dims)):
        got, threads = oracle.mttkrp_all_cores(dims, inds, vals, facs, n)
        assert threads >= 1
        np.testing.assert_allclose(got, oracle.mttkrp(dims, inds, vals, facs, n), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(got, _unfold(x, n) @ _khatri_rao_all_but(facs, n), rtol=1e-11, atol=1e-12)
    bad = [a.copy() for a in inds]
    bad[0][3] = dims[0]
    with pytest.raises(RuntimeError):
        oracle.mttkrp_all_cores(dims, bad, vals, facs, 1)


@pytest.mark.parametrize("dims", [(5, 4, 3), (3, 4, 2, 5), (2, 3, 4, 2, 3)])
def test_fp64_factor_variant_against_the_dense_definition(oracle, dims):
    """oracle.mttkrp_f64 (fp64 factor matrices, nothing widened but the value) against Eq. 4 with factors whose
    values need all 53 mantissa bits; it must differ from the fp32-factor oracle fed the rounded factors (so a
    variant that narrowed its factors would fail the first check), and agree with it on fp32-valued factors."""
    rng = np.random.default_rng(97 + len(dims))
    inds, vals = _random_coo(rng, dims, max(1, int(0.5 * np.prod(dims))))
    facs = [rng.uniform(0.1, 1, size=(d, 5)) for d in dims]
    x = _dense(dims, inds, vals)
    for n in range(len(dims)):
        want = _unfold(x, n) @ _khatri_rao_all_but(facs, n)
        got = oracle.mttkrp_f64(dims, inds, vals, facs, n)
        assert got.dtype == np.float64 and got.shape == (dims[n], 5)
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-14)
        narrowed = oracle.mttkrp(dims, inds, vals, [f.astype(np.float32) for f in facs], n)
        assert np.max(np.abs(narrowed - want)) > 1e-9
        f32 = [f.astype(np.float32) for f in facs]
        np.testing.assert_array_equal(oracle.mttkrp_f64(dims, inds, vals, [f.astype(np.float64) for f in f32], n),
                                      oracle.mttkrp(dims, inds, vals, f32, n))
