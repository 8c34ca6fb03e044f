"""TEST INFRASTRUCTURE ONLY: plain CPU oracle of one CPD-ALS iteration (Section II-B, Eq. 1-3, Algorithm
"CPD-ALS").  Nothing in the product path may import this file; it shares no code with the GPU library.

One iteration, in the algorithm's order and notation, for an order-N tensor with factor matrices A_1..A_N:

    for n = 1..N:   A_n <- X_(n) (Khatri-Rao of the other factors) (Hadamard_{m != n} A_m^T A_m)^+
    normalise the columns of every A_n and store the norms in lambda

The first product is the mode-n MTTKRP (Section II-C, Eq. 4), evaluated here per nonzero in fp64 with numpy
(Eq. 7); ^+ is the Moore-Penrose pseudo-inverse (numpy.linalg.pinv).  Everything is fp64.

Readings (the paper leaves them open): the "*" between the Gram matrices is the element-wise product (the normal
equations of Eq. 2), whatever the prose under Eq. 3 calls it; the column normalisation step of Algorithm "CPD-ALS" is applied once, at
the end of the iteration, where the algorithm lists it; the norm is the 2-norm; lambda_r is the product over the modes of the
r-th column norms, so that [[lambda; A_1..A_N]] is the same model as the unnormalised factors; a zero column is
left as it is (norm taken as 1).
"""
from __future__ import annotations

import numpy as np


def mttkrp(dims, inds, vals, factors, mode):
    """fp64 mode-`mode` MTTKRP from fp64 factor matrices: M[i_n] += v * prod_{m != n} A_m[i_m]."""
    rank = factors[(mode + 1) % len(dims)].shape[1]
    prod = np.repeat(np.asarray(vals, dtype=np.float64)[:, None], rank, axis=1)
    for m in range(len(dims)):
        if m != mode:
            prod = prod * np.asarray(factors[m], dtype=np.float64)[np.asarray(inds[m], dtype=np.int64)]
    out = np.zeros((dims[mode], rank))
    np.add.at(out, np.asarray(inds[mode], dtype=np.int64), prod)
    return out


def gram(a):
    """fp64 Gram matrix A^T A of a factor matrix: the R x R matrices whose Hadamard product Eq. 3 inverts."""
    a = np.asarray(a, dtype=np.float64)
    return a.T @ a


def als_iteration(dims, inds, vals, factors):
    """One iteration of Algorithm "CPD-ALS".  factors: list of [dims[m], R] arrays (any float dtype).
    Returns (new fp64 factors with unit-norm columns, lambda)."""
    order = len(dims)
    a = [np.array(f, dtype=np.float64) for f in factors]
    rank = a[0].shape[1]
    for n in range(order):
        m_n = mttkrp(dims, inds, vals, a, n)
        v = np.ones((rank, rank))
        for m in range(order):
            if m != n:
                v = v * (a[m].T @ a[m])
        a[n] = m_n @ np.linalg.pinv(v)
    lam = np.ones(rank)
    for n in range(order):
        norms = np.sqrt((a[n] * a[n]).sum(axis=0))
        norms = np.where(norms > 0, norms, 1.0)
        a[n] = a[n] / norms
        lam = lam * norms
    return a, lam


def model_values(inds, factors, lam):
    """Values of the model [[lambda; A_1..A_N]] (Eq. 1) at the given coordinates."""
    p = np.repeat(np.asarray(lam, dtype=np.float64)[None, :], len(inds[0]), axis=0)
    for m, f in enumerate(factors):
        p = p * np.asarray(f, dtype=np.float64)[np.asarray(inds[m], dtype=np.int64)]
    return p.sum(axis=1)


def fit(dims, inds, vals, factors, lam):
    """1 - ||X - model|| / ||X|| for a sparse X with distinct coordinates, without forming the model densely:
    ||X - model||^2 = ||X||^2 - 2 <X, model> + ||model||^2, the inner product summed over the nonzeros and
    ||model||^2 = sum_{r,s} lambda_r lambda_s prod_m (A_m^T A_m)[r, s]."""
    vals = np.asarray(vals, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    inner = float((vals * model_values(inds, factors, lam)).sum())
    g = np.outer(lam, lam)
    for f in factors:
        f = np.asarray(f, dtype=np.float64)
        g = g * (f.T @ f)
    x2 = float((vals * vals).sum())
    res2 = max(x2 - 2.0 * inner + float(g.sum()), 0.0)
    return 1.0 - np.sqrt(res2) / np.sqrt(x2)
