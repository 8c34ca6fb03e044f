"""GPU parity of the fp64 entry point (hbcsf_mttkrp_f64) against the oracle's fp64-factor form, element by element."""
import numpy as np
import pytest

import gpu_util as GU
from paper_1904_03329_amd import HbcsfTensor, binding as B

pytestmark = pytest.mark.gpu


def _skewed(rng, dims, nnz, a=1.3):
    inds = []
    for d in dims:
        w = 1.0 / np.arange(1, d + 1) ** a
        inds.append(rng.permutation(d)[rng.choice(d, size=nnz, p=w / w.sum())].astype(np.uint32))
    key = np.zeros(nnz, dtype=np.int64)
    for d, x in zip(dims, inds):
        key = key * d + x
    _, first = np.unique(key, return_index=True)
    first = rng.permutation(first)
    return [x[first] for x in inds], rng.uniform(-1, 1, size=first.shape[0]).astype(np.float32)


def _factors64(rng, dims, rank):
    """Values that need the whole fp64 mantissa, so a path that narrowed them would miss the bar by 1e5."""
    return [rng.uniform(0, 1, size=(d, rank)) for d in dims]


def _check_all_modes(oracle, dims, inds, vals, facs, what, **kw):
    outs, stats = GU.gpu_mttkrp_all_modes(dims, inds, vals, facs, **kw)
    worst = 0.0
    for mode, got in enumerate(outs):
        assert got.dtype == np.float64
        want = oracle.mttkrp_f64(dims, inds, vals, facs, mode)
        worst = max(worst, GU.assert_close(got, want, f"{what} mode {mode}", tol=GU.REL_TOL_F64))
    print(f"{what}: max|diff|/max|M| = {worst:.2e}", flush=True)
    return stats


@pytest.mark.parametrize("rank", [16, 32, 64])
@pytest.mark.parametrize("dims,nnz", [((3000, 700, 90), 60_000), ((900, 300, 40, 25), 50_000),
                                      ((600, 200, 30, 12, 8), 50_000)])
def test_ranks_and_orders(oracle, dims, nnz, rank):
    rng = np.random.default_rng(rank * 10 + len(dims))
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors64(rng, dims, rank)
    print("f64 ranks_and_orders", dims, vals.shape[0], rank, flush=True)
    stats = _check_all_modes(oracle, dims, inds, vals, facs, f"f64 R={rank} order={len(dims)}")
    assert all(s["group_nnz"][2] > 0 for s in stats)


@pytest.mark.parametrize("opts", [dict(group_mask=4), dict(group_mask=1), dict(group_mask=2), dict(fiber_threshold=8),
                                  dict(fiber_threshold=16, tune_ts=256), dict(mode_order_policy=1),
                                  dict(hybrid_granularity=1), dict(coo_row_flags=1), dict(mid_blocking=4),
                                  dict(tune_steps=4), dict(tune_ts=100_000)])
@pytest.mark.parametrize("dims,nnz", [((5000, 400, 60), 120_000), ((2000, 100, 30, 12), 90_000)])
def test_build_options_do_not_change_the_result(oracle, dims, nnz, opts):
    rng = np.random.default_rng(len(dims) + 11)
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors64(rng, dims, 32)
    print("f64 options", dims, vals.shape[0], opts, flush=True)
    _check_all_modes(oracle, dims, inds, vals, facs, f"f64 {opts}", **opts)


def test_rank_16_kernel_variants(oracle):
    """Rank 16 in fp64 is the 8-lanes-per-row mapping: its held-to-128-registers B-CSF variant and the dense
    fiber-row gather (a tuning variant) are instantiated for doubles too."""
    rng = np.random.default_rng(5)
    dims = (4000, 500, 80)
    inds, vals = _skewed(rng, dims, 150_000)
    facs = _factors64(rng, dims, 16)
    for kw in (dict(), dict(tune_dense=1), dict(tune_dense=1, group_mask=4)):
        print("f64 rank 16", kw, flush=True)
        _check_all_modes(oracle, dims, inds, vals, facs, f"f64 R=16 {kw}", **kw)


@pytest.mark.parametrize("dims,nnz,a", [((200, 5, 30_000), 400_000, 0.2), ((40, 9000, 11_000), 300_000, 0.6),
                                        ((3, 50, 4000), 10_007, 0.0), ((7, 5, 3), 60, 0.0)])
def test_heavy_slices_long_fibers_and_tiny_tensors(oracle, dims, nnz, a):
    """Slices far above the work unit (merged with fp64 atomic adds), fibers above T_f, a ragged last unit, and a
    tensor smaller than one unit."""
    rng = np.random.default_rng(nnz % 1000 + len(dims))
    inds, vals = _skewed(rng, dims, nnz, a=a)
    facs = _factors64(rng, dims, 32)
    print("f64 heavy", dims, vals.shape[0], flush=True)
    _check_all_modes(oracle, dims, inds, vals, facs, f"f64 heavy {dims}")
    _check_all_modes(oracle, dims, inds, vals, facs, f"f64 heavy {dims} plain B-CSF", group_mask=4, tune_ts=512)


def test_factor_matrix_above_4GiB(oracle, synth):
    """A factor matrix of 17 M rows x 32 doubles exceeds 4 GiB: the 64-bit-offset instantiations in fp64.  Every
    non-empty output row against the oracle (fp32-valued factors here: the rows-only oracle takes fp32 factors),
    every other row exactly zero."""
    import torch

    dims, nnz, alpha = (17_000_000, 17_000_000, 100), 1_200_000, (1.05, 1.05, 0.0)
    t = synth.tensor(dims, nnz, alpha, seed=777)
    facs = synth.factors(t.dims, 32, seed=778)
    print("f64 wide", t.dims, t.nnz, flush=True)
    ht = HbcsfTensor(t.dims, t.inds, t.vals).to_device()
    dfacs = [torch.from_numpy(f).cuda().double() for f in facs]
    for mode in range(t.order):
        out = torch.full((t.dims[mode], 32), float("nan"), dtype=torch.float64, device="cuda")
        ht.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        rows = np.unique(t.inds[mode])
        want = oracle.mttkrp_rows(t.dims, t.inds, t.vals, facs, mode, rows)
        drows = torch.from_numpy(rows.astype(np.int64)).cuda()
        rel = GU.assert_close(out[drows].cpu().numpy(), want, f"f64 wide mode {mode}", tol=GU.REL_TOL_F64)
        out[drows] = 0.0
        assert int(torch.count_nonzero(out)) == 0 and bool(torch.isfinite(out).all()), "an empty slice's row is not zero"
        print(f"f64 wide mode {mode}: {rows.size} non-empty rows, max|diff|/max|M| = {rel:.2e}", flush=True)
        del out
    ht.close()


def test_cfg2_every_element(oracle, synth):
    """The 3-order benchmark workload with dense short modes at full size, all modes, every element."""
    t, facs, rank = synth.workload("cfg2")
    facs64 = [f.astype(np.float64) + 1e-9 * np.cos(np.arange(f.size, dtype=np.float64)).reshape(f.shape) for f in facs]
    print("f64 cfg2", t.dims, t.nnz, rank, flush=True)
    _check_all_modes(oracle, t.dims, t.inds, t.vals, facs64, "f64 cfg2")


def test_cfg3_every_element(oracle, synth):
    """The 100 M-nonzero power-law benchmark workload at full size in fp64: slices of up to 11.6 M nonzeros merged with
    fp64 atomic adds, all modes, every element."""
    t, facs, rank = synth.workload("cfg3")
    facs64 = [f.astype(np.float64) + 1e-9 * np.cos(np.arange(f.size, dtype=np.float64)).reshape(f.shape) for f in facs]
    print("f64 cfg3", t.dims, t.nnz, rank, flush=True)
    _check_all_modes(oracle, t.dims, t.inds, t.vals, facs64, "f64 cfg3")


def test_argument_errors():
    import torch

    rng = np.random.default_rng(3)
    dims = (50, 40, 30)
    inds, vals = _skewed(rng, dims, 2000)
    t = HbcsfTensor(dims, inds, vals).to_device()
    for rank in (8, 128, 24):
        facs = [torch.zeros((d, rank), dtype=torch.float64, device="cuda") for d in dims]
        with pytest.raises(B.HbcsfError):
            t.mttkrp(0, facs)
    mixed = [torch.zeros((d, 32), dtype=torch.float64 if m else torch.float32, device="cuda") for m, d in enumerate(dims)]
    with pytest.raises(ValueError):
        t.mttkrp(0, [None, mixed[1].float(), mixed[2]])
    t.close()
    single = HbcsfTensor(dims, inds, vals, single_representation=1).to_device()
    facs = [torch.zeros((d, 32), dtype=torch.float64, device="cuda") for d in dims]
    with pytest.raises(B.HbcsfError):
        single.mttkrp(1, facs)
    single.close()
