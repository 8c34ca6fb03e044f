"""GPU parity of the CPD-ALS iteration (Section II-B, Algorithm "CPD-ALS") against the numpy fp64 oracle.

Bar: the device computes the MTTKRP and the two dense passes in fp32, the oracle everything in fp64.  A
relative error e in M or in a Gram matrix reaches the updated factor amplified by at most the condition
number of the Hadamard product V of Gram matrices, so the bound used is
    max |A_gpu - A_oracle| <= 1e-5 * max(cond(V), 10) * max |A_oracle|
per factor (columns have unit norm), the same for lambda relative to its largest entry, and 1e-5 absolute
for the fit.  The starting factors are uniform in (-1, 1), which keeps cond(V) near 1 in the first iteration.
"""
import numpy as np
import pytest

from oracle import cpd_als

pytestmark = pytest.mark.gpu


def _random_tensor(rng, dims, nnz):
    total = int(np.prod([float(d) for d in dims]))
    flat = rng.choice(total, size=min(nnz, total), replace=False)
    inds = []
    for d in reversed(dims):
        inds.append((flat % d).astype(np.uint32))
        flat = flat // d
    inds = inds[::-1]
    vals = rng.uniform(0.1, 1.0, size=len(inds[0])).astype(np.float32)
    return inds, vals


def _worst_cond(dims, inds, vals, facs):
    """Largest condition number of the Hadamard products the oracle inverts during the iteration."""
    a = [np.array(f, dtype=np.float64) for f in facs]
    worst = 1.0
    for n in range(len(dims)):
        v = np.ones((a[0].shape[1],) * 2)
        for m in range(len(dims)):
            if m != n:
                v = v * (a[m].T @ a[m])
        worst = max(worst, np.linalg.cond(v))
        a[n] = cpd_als.mttkrp(dims, inds, vals, a, n) @ np.linalg.pinv(v)
    return worst


def _run_gpu(dims, inds, vals, facs, rank, iterations=1, keep=False, lazy=False):
    import torch
    from paper_1904_03329_amd import CpdAls, HbcsfTensor

    t = HbcsfTensor(dims, inds, vals).to_device()
    als = CpdAls(t, rank)
    dfacs = [torch.from_numpy(np.ascontiguousarray(f)).cuda() for f in facs]
    fits = []
    for it in range(iterations):
        fits.append(als.iteration(dfacs, keep_grams=keep and it > 0, lazy=lazy))
    if lazy:
        als.normalise(dfacs)
    torch.cuda.synchronize()
    out = [f.cpu().numpy() for f in dfacs]
    lam = als.lam.cpu().numpy()
    phases = als.phase_ms()
    als.close()
    t.close()
    return out, lam, fits, phases


def _check(dims, inds, vals, facs, rank, iterations=1, keep=False, lazy=False):
    got, lam, fits, _ = _run_gpu(dims, inds, vals, facs, rank, iterations, keep, lazy)
    want = [np.array(f, dtype=np.float64) for f in facs]
    cond = 1.0
    for _ in range(iterations):
        cond = max(cond, _worst_cond(dims, inds, vals, want))
        want, want_lam = cpd_als.als_iteration(dims, inds, vals, want)
    tol = 1e-5 * max(cond, 10.0)
    for m, (g, w) in enumerate(zip(got, want)):
        assert np.all(np.isfinite(g))
        err = np.max(np.abs(g - w)) / np.max(np.abs(w))
        assert err <= tol, f"factor {m}: {err:.2e} > {tol:.2e} (cond {cond:.1f})"
    assert np.max(np.abs(lam - want_lam)) <= tol * np.max(np.abs(want_lam))
    assert abs(fits[-1] - cpd_als.fit(dims, inds, vals, want, want_lam)) <= max(tol, 1e-5)
    return fits


@pytest.mark.parametrize("rank", [32, 8, 16, 64, 128])
def test_one_iteration_third_order(rank):
    rng = np.random.default_rng(100 + rank)
    dims = (1000, 333, 77)          # several 32-row blocks, ragged tails, one dimension below a block pair
    inds, vals = _random_tensor(rng, dims, 40000)
    facs = [rng.uniform(-1, 1, size=(d, rank)).astype(np.float32) for d in dims]
    _check(dims, inds, vals, facs, rank)


@pytest.mark.parametrize("rank", [32, 16])
def test_one_iteration_fourth_order(rank):
    rng = np.random.default_rng(200 + rank)
    dims = (130, 65, 31, 9)
    inds, vals = _random_tensor(rng, dims, 30000)
    facs = [rng.uniform(-1, 1, size=(d, rank)).astype(np.float32) for d in dims]
    _check(dims, inds, vals, facs, rank)


def test_one_iteration_fifth_order():
    rng = np.random.default_rng(555)
    dims = (70, 33, 17, 9, 5)
    inds, vals = _random_tensor(rng, dims, 30000)
    facs = [rng.uniform(-1, 1, size=(d, 16)).astype(np.float32) for d in dims]
    _check(dims, inds, vals, facs, 16)


def test_three_iterations_reuse_gram_matrices():
    rng = np.random.default_rng(300)
    dims = (400, 300, 200)
    inds, vals = _random_tensor(rng, dims, 60000)
    facs = [rng.uniform(-1, 1, size=(d, 32)).astype(np.float32) for d in dims]
    fits_keep = _check(dims, inds, vals, facs, 32, iterations=3, keep=True)
    fits_fresh = _check(dims, inds, vals, facs, 32, iterations=3, keep=False)
    np.testing.assert_allclose(fits_keep, fits_fresh, atol=1e-5)
    assert fits_keep[2] >= fits_keep[1] - 1e-6 >= fits_keep[0] - 2e-6      # ALS never lowers the fit


@pytest.mark.parametrize("rank", [32, 16])
@pytest.mark.parametrize("dims", [(1000, 333, 77), (130, 65, 31, 9)])
def test_put_off_normalisation(rank, dims):
    """HBCSF_ALS_LAZY_NORMALISATION: three iterations whose closing normalisation is put off (at R = 32 the product
    kernel then also forms the new factor's Gram matrix), hbcsf_als_normalise at the end; factors, lambda and every
    iteration's fit as the oracle's.  Then an ordinary iteration on a state that still has norms pending."""
    import torch
    from paper_1904_03329_amd import CpdAls, HbcsfTensor

    rng = np.random.default_rng(4000 + rank + len(dims))
    inds, vals = _random_tensor(rng, dims, 40000)
    facs = [rng.uniform(-1, 1, size=(d, rank)).astype(np.float32) for d in dims]
    fits_lazy = _check(dims, inds, vals, facs, rank, iterations=3, keep=True, lazy=True)
    fits_eager = _check(dims, inds, vals, facs, rank, iterations=3, keep=True, lazy=False)
    np.testing.assert_allclose(fits_lazy, fits_eager, atol=1e-5)
    # two put-off iterations, then one that normalises by itself: same as three ordinary ones
    t = HbcsfTensor(dims, inds, vals).to_device()
    als = CpdAls(t, rank)
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    als.iteration(dfacs, lazy=True)
    als.iteration(dfacs, keep_grams=True, lazy=True)
    fit = als.iteration(dfacs, keep_grams=True)
    want = [f.astype(np.float64) for f in facs]
    for _ in range(3):
        want, want_lam = cpd_als.als_iteration(dims, inds, vals, want)
    for g, w in zip(dfacs, want):
        assert np.max(np.abs(g.cpu().numpy() - w)) <= 2e-4 * np.max(np.abs(w))
    np.testing.assert_allclose(torch.sqrt((dfacs[1].double() ** 2).sum(dim=0)).cpu().numpy(), 1.0, atol=1e-4)
    assert abs(fit - fits_eager[2]) <= 1e-5
    als.close()
    t.close()


def test_recovers_an_exact_low_rank_tensor():
    """All entries of a rank-8 model are stored, so the fit of the true factors is 1 and stays there."""
    rng = np.random.default_rng(400)
    dims = (40, 30, 20)
    rank = 8
    true = [rng.uniform(0.2, 1, size=(d, rank)) for d in dims]
    grid = np.meshgrid(*[np.arange(d) for d in dims], indexing="ij")
    inds = [g.ravel().astype(np.uint32) for g in grid]
    vals = cpd_als.model_values(inds, true, np.ones(rank)).astype(np.float32)
    got, lam, fits, _ = _run_gpu(dims, inds, vals, [f.astype(np.float32) for f in true], rank)
    # the fit is 1 - sqrt(||X||^2 - 2<X, model> + ||model||^2) / ||X||: the three terms cancel, so fp32 rounding
    # of the MTTKRP (relative 1e-6) limits its resolution near 1 to about sqrt(1e-6)
    assert fits[0] > 1 - 3e-3
    model = cpd_als.model_values(inds, got, lam)
    assert np.max(np.abs(model - vals)) <= 1e-3 * np.max(np.abs(vals))


def test_config1_shape(synth):
    t, _, rank = synth.workload("cfg1")
    rng = np.random.default_rng(500)
    facs = [rng.uniform(-1, 1, size=(d, rank)).astype(np.float32) for d in t.dims]
    _check(t.dims, t.inds, t.vals, facs, rank)


def test_config2_shape_at_one_tenth(synth):
    """One iteration on the second workload's index laws at R = 32, scaled to 500 000 nonzeros so that the numpy
    oracle finishes in seconds (10 000-row factors still span many wavefront chunks of the dense kernels)."""
    t, _, rank = synth.workload("cfg2", scale=0.1)
    rng = np.random.default_rng(700)
    facs = [rng.uniform(-1, 1, size=(d, rank)).astype(np.float32) for d in t.dims]
    _check(t.dims, t.inds, t.vals, facs, rank)


def test_factor_matrix_above_4GiB(synth):
    """A 34 M-row factor matrix at R = 32 is 4.35 GB: the Gram and product kernels then index beyond 2^32 bytes,
    and the MTTKRPs of the other modes gather from it with 64-bit offsets.  One iteration against the oracle."""
    with open("/proc/meminfo") as f:
        avail = [int(l.split()[1]) for l in f if l.startswith("MemAvailable:")][0] / (1 << 20)
    if avail < 64:
        pytest.skip(f"the fp64 numpy oracle holds several 8.7 GB matrices: needs about 64 GiB of host memory, "
                    f"{avail:.0f} GiB available")
    dims, rank = (34_000_000, 300, 40), 32
    t = synth.tensor(dims, 2_000_000, (1.05, 1.1, 0.0), seed=900)
    vals = (0.1 + 0.45 * (t.vals + 1.0)).astype(np.float32)      # positive, as in the other cases
    facs = [synth.uniform((d, rank), 900 + m, -1.0, 1.0) for m, d in enumerate(dims)]
    print("als wide", dims, t.nnz, flush=True)
    _check(dims, t.inds, vals, facs, rank)


def test_run_until_the_fit_settles():
    """The outer loop on a noisy low-rank tensor: stops by the tolerance, before the iteration cap, at the fit
    the oracle reaches with the same number of iterations."""
    import torch
    from paper_1904_03329_amd import CpdAls, HbcsfTensor

    rng = np.random.default_rng(800)
    dims, rank = (60, 50, 40), 8
    true = [rng.uniform(0, 1, size=(d, rank)) for d in dims]
    grid = np.meshgrid(*[np.arange(d) for d in dims], indexing="ij")
    inds = [g.ravel().astype(np.uint32) for g in grid]
    vals = (cpd_als.model_values(inds, true, np.ones(rank)) + 0.05 * rng.normal(size=len(inds[0]))).astype(np.float32)
    facs = [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]
    t = HbcsfTensor(dims, inds, vals).to_device()
    als = CpdAls(t, rank)
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    done, fit = als.run(dfacs, max_iterations=200, tolerance=1e-4)
    assert 2 <= done < 200 and fit > 0.8
    want = [f.astype(np.float64) for f in facs]
    for _ in range(done):
        want, lam = cpd_als.als_iteration(dims, inds, vals, want)
    assert abs(fit - cpd_als.fit(dims, inds, vals, want, lam)) < 2e-3
    als.close()
    t.close()


def test_argument_errors():
    import torch
    from paper_1904_03329_amd import HbcsfTensor, binding as B

    rng = np.random.default_rng(600)
    dims = (50, 40, 30)
    inds, vals = _random_tensor(rng, dims, 500)
    t = HbcsfTensor(dims, inds, vals)
    ws = torch.empty(B.als_workspace_bytes(t.handle, 32), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.HbcsfError) as e:
        B.als_create(t.handle, 32, ws.data_ptr(), ws.numel())
    assert e.value.code == -4                                  # not uploaded
    t.to_device()
    with pytest.raises(B.HbcsfError) as e:
        B.als_create(t.handle, 24, ws.data_ptr(), ws.numel())
    assert e.value.code == -1
    with pytest.raises(B.HbcsfError) as e:
        B.als_create(t.handle, 32, ws.data_ptr(), 1024)
    assert e.value.code == -3
    a = B.als_create(t.handle, 32, ws.data_ptr(), ws.numel())
    f = [torch.zeros((d, 32), device="cuda") for d in dims]
    with pytest.raises(B.HbcsfError) as e:
        B.als_iteration(a, [f[0].data_ptr(), 0, f[2].data_ptr()])
    assert e.value.code == -1
    with pytest.raises(B.HbcsfError) as e:
        B.als_iteration(a, [x.data_ptr() for x in f], flags=8)
    assert e.value.code == -1
    B.als_free(a)
    t.close()
