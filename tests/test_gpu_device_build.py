"""The device-side format builder against the host builder (array for array, bit for bit), against the
CPU walks of tests/format_walk.py, and end to end against the MTTKRP oracle."""
import numpy as np
import pytest

import format_walk as FW
import gpu_util as GU
from paper_1904_03329_amd import binding as B

pytestmark = pytest.mark.gpu


def _device_tensor(dims, inds, vals, **opts):
    import torch
    from paper_1904_03329_amd import HbcsfTensor

    di = [torch.from_numpy(np.ascontiguousarray(x, dtype=np.uint32).view(np.int32)).cuda() for x in inds]
    dv = torch.from_numpy(np.ascontiguousarray(vals, dtype=np.float32)).cuda()
    return HbcsfTensor.from_device_coo(dims, di, dv, **opts)


def _arrays(h, order, modes=None):
    out = {}
    for mode in (range(order) if modes is None else modes):
        for aid in (B.ARR_OWNED_BITS, B.ARR_COO_BITS, B.ARR_COO_PTR):
            out[(mode, aid)] = B.host_array(h, mode, 0, 0, aid)
        for g in range(3):
            for lvl in range(order):
                for aid in (B.ARR_IND, B.ARR_PTR, B.ARR_RUNFIRST):
                    try:
                        out[(mode, g, lvl, aid)] = B.host_array(h, mode, g, lvl, aid)
                    except B.HbcsfError:
                        pass
            out[(mode, g, "val")] = B.host_array(h, mode, g, 0, B.ARR_VAL).view(np.uint32)
    return out


def assert_same_format(dims, inds, vals, **opts):
    """Builds on the host and on the device; every array and every statistic must agree."""
    from paper_1904_03329_amd import HbcsfTensor

    order = len(dims)
    host = HbcsfTensor(dims, inds, vals, **opts)
    dev = _device_tensor(dims, inds, vals, **opts)
    assert B.device_bytes(dev.handle) == B.device_bytes(host.handle)
    with pytest.raises(B.HbcsfError):
        B.host_array(dev.handle, 0, 0, 0, B.ARR_VAL)          # no host copy yet
    B.download(dev.handle)
    modes = [0] if opts.get("single_representation") else list(range(order))   # one stored tree / one per mode
    for mode in modes:
        sh, sd = host.stats(mode), dev.stats(mode)
        sh.pop("build_seconds"), sd.pop("build_seconds")
        assert sh == sd, f"mode {mode}: statistics differ"
    ah, ad = _arrays(host.handle, order, modes), _arrays(dev.handle, order, modes)
    assert ah.keys() == ad.keys()
    for k in ah:
        assert np.array_equal(ah[k], ad[k]), f"array {k} differs"
    host.close()
    return dev


def _random(rng, dims, nnz, distinct=True):
    inds = [rng.integers(0, d, nnz).astype(np.uint32) for d in dims]
    if distinct:
        key = np.zeros(nnz, dtype=np.int64)
        for i, d in zip(inds, dims):
            key = key * d + i
        _, keep = np.unique(key, return_index=True)
        keep.sort()
        inds = [i[keep] for i in inds]
    vals = rng.uniform(-1, 1, len(inds[0])).astype(np.float32)
    return inds, vals


def _skewed(rng, dims, nnz, a=1.3):
    inds = []
    for d in dims:
        p = 1.0 / np.arange(1, d + 1) ** a
        inds.append(rng.permutation(d)[rng.choice(d, size=nnz, p=p / p.sum())].astype(np.uint32))
    key = np.zeros(nnz, dtype=np.int64)
    for i, d in zip(inds, dims):
        key = key * d + i
    _, keep = np.unique(key, return_index=True)
    keep.sort()
    return [i[keep] for i in inds], rng.uniform(-1, 1, keep.size).astype(np.float32)


def test_cfg1_arrays_walks_and_mttkrp(oracle, synth):
    import torch

    t, facs, rank = synth.workload("cfg1")
    dev = assert_same_format(t.dims, t.inds, t.vals)
    for mode in range(t.order):
        fmt = FW.read_mode(dev.handle, mode, t.order)
        want = oracle.mttkrp(t.dims, t.inds, t.vals, facs, mode)
        got = FW.walk_algorithms(fmt, facs, t.dims[mode], rank)
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-9 * np.abs(want).max())
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    for mode in range(t.order):
        out = dev.mttkrp(mode, dfacs)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), oracle.mttkrp(t.dims, t.inds, t.vals, facs, mode), f"cfg1 mode {mode}")
    dev.close()


@pytest.mark.parametrize("opts", [dict(), dict(fiber_threshold=8), dict(fiber_threshold=16), dict(group_mask=4),
                                  dict(group_mask=1), dict(group_mask=2), dict(mode_order_policy=1),
                                  dict(mode_order_policy=2), dict(coo_row_flags=1), dict(mid_blocking=3),
                                  dict(mid_blocking=5, fiber_threshold=16), dict(hybrid_granularity=1),
                                  dict(hybrid_granularity=1, fiber_threshold=8),
                                  dict(hybrid_granularity=1, fiber_threshold=16, mid_blocking=3),
                                  dict(hybrid_granularity=1, group_mask=2, mode_order_policy=1)])
@pytest.mark.parametrize("dims,nnz", [((5000, 400, 60), 120_000), ((2000, 100, 30, 12), 90_000),
                                      ((1500, 80, 20, 9, 6), 90_000)])
def test_same_arrays_as_the_host_builder(dims, nnz, opts):
    rng = np.random.default_rng(len(dims) * 1000 + nnz)
    inds, vals = _skewed(rng, dims, nnz)
    dev = assert_same_format(dims, inds, vals, **opts)
    if opts.get("hybrid_granularity") and opts.get("fiber_threshold", 64) <= 16:
        # the per-fiber choice really splits slices of these tensors: nonzeros move from the CSF to the CSL group
        from paper_1904_03329_amd import HbcsfTensor
        plain = HbcsfTensor(dims, inds, vals, **{k: v for k, v in opts.items() if k != "hybrid_granularity"})
        moved = [dev.stats(m)["group_nnz"][1] - plain.stats(m)["group_nnz"][1] for m in range(len(dims))]
        plain.close()
        assert max(moved) > 0 and min(moved) >= 0, moved
    dev.close()


@pytest.mark.parametrize("dims,nnz", [((3000, 700, 90), 200_000), ((900, 300, 40, 25), 150_000),
                                      ((600, 200, 30, 12, 8), 120_000)])
def test_single_representation(oracle, dims, nnz):
    """single_representation = 1 built on the device: mode 0's plain B-CSF tree only, equal to the host's, and every
    mode's MTTKRP from it against the oracle (rank 32)."""
    import torch

    rng = np.random.default_rng(len(dims) * 13 + 1)
    inds, vals = _skewed(rng, dims, nnz)
    dev = assert_same_format(dims, inds, vals, single_representation=1)
    facs = [rng.uniform(0, 1, size=(d, 32)).astype(np.float32) for d in dims]
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    for mode in range(len(dims)):
        out = torch.full((dims[mode], 32), float("nan"), dtype=torch.float32, device="cuda")
        dev.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), oracle.mttkrp(dims, inds, vals, facs, mode), f"single, device-built, mode {mode}")
    with pytest.raises(B.HbcsfError) as e:
        _device_tensor(dims, inds, vals, single_representation=1, group_mask=1)
    assert e.value.code == -1
    dev.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_small_tensors(oracle, seed):
    """Random small tensors (duplicates allowed in some) with the build options drawn at random: both builders give the
    same arrays, and the MTTKRP from the device-built handle matches the oracle."""
    import torch

    rng = np.random.default_rng(7000 + seed)
    order = 3 + seed % 3
    dims = tuple(int(rng.integers(1, 200 if order < 5 else 40)) for _ in range(order))
    nnz = int(rng.integers(1, 3000))
    inds, vals = _random(rng, dims, nnz, distinct=bool(seed % 4))
    rank = [8, 16, 32][seed % 3]
    opts = dict(fiber_threshold=int(rng.choice([8, 16, 32, 64])), mode_order_policy=int(rng.integers(0, 3)),
                group_mask=int(rng.choice([0, 0, 1, 2, 4])), hybrid_granularity=int(rng.integers(0, 2)),
                coo_row_flags=int(rng.integers(0, 2)), mid_blocking=int(rng.choice([0, 0, 2, 3])))
    print("random", dims, nnz, rank, opts, flush=True)
    dev = assert_same_format(dims, inds, vals, **opts)
    facs = [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    for mode in range(order):
        out = dev.mttkrp(mode, dfacs)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), oracle.mttkrp(dims, inds, vals, facs, mode), f"seed {seed} mode {mode}")
    dev.close()


def test_duplicates_keep_their_input_order():
    """Equal coordinates are not merged; the sort is stable, so their values stay in input order."""
    rng = np.random.default_rng(42)
    dims = (30, 20, 10)
    inds, vals = _random(rng, dims, 4000, distinct=False)
    assert_same_format(dims, inds, vals).close()


def test_empty_tensor():
    import torch

    dims = (9, 8, 7)
    empty = [np.zeros(0, dtype=np.uint32) for _ in dims]
    dev = assert_same_format(dims, empty, np.zeros(0, dtype=np.float32))
    facs = [torch.ones((d, 8), device="cuda") for d in dims]
    for mode in range(3):
        out = torch.full((dims[mode], 8), float("nan"), device="cuda")
        dev.mttkrp(mode, facs, out)
        torch.cuda.synchronize()
        assert float(out.abs().max()) == 0.0
    dev.close()


def test_degenerate_shapes():
    one = (np.array([3], dtype=np.uint32), np.array([0], dtype=np.uint32), np.array([5], dtype=np.uint32))
    assert_same_format((7, 1, 9), one, np.array([2.5], dtype=np.float32)).close()
    # one heavy slice spanning many runs, one long fiber
    n = 1000
    inds = [np.zeros(n, dtype=np.uint32), np.zeros(n, dtype=np.uint32), np.arange(n, dtype=np.uint32)]
    assert_same_format((2, 1, n), inds, np.ones(n, dtype=np.float32)).close()
    # already sorted input, large sparse dimensions
    inds = [np.arange(n, dtype=np.uint32) * 1000, np.arange(n, dtype=np.uint32) * 7, np.arange(n, dtype=np.uint32)]
    assert_same_format((1_000_000, 7_000, n), inds, np.ones(n, dtype=np.float32)).close()


@pytest.mark.parametrize("dims", [(100_000, 90_000, 80_000, 70_000), (2_000_000_000, 1_500_000_000, 3_000),
                                  (100_000, 90_000, 80_000, 700, 60)])
def test_wide_coordinates_sort_in_two_passes(oracle, dims):
    """Packed coordinates above 64 bits (68, 74 and, at order 5, 67 here) take the 128-bit key path of both builders."""
    import torch

    rng = np.random.default_rng(len(dims))
    nnz = 30_000
    inds = [rng.integers(0, d, nnz).astype(np.uint32) for d in dims]
    for x in inds:                                              # repeated indices so that slices and fibers exist
        x[nnz // 2:] = x[rng.integers(0, 200, nnz - nnz // 2)]
    vals = rng.uniform(-1, 1, nnz).astype(np.float32)
    dev = assert_same_format(dims, inds, vals)
    mode = len(dims) - 1                                        # the shortest mode: a dense check is affordable
    rank = 8
    facs = [None if d > 1_000_000 else rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]
    if all(f is not None for f in facs):
        dfacs = [torch.from_numpy(f).cuda() for f in facs]
        out = dev.mttkrp(mode, dfacs)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), oracle.mttkrp(dims, inds, vals, facs, mode), "wide keys")
    dev.close()


def test_cfg2_full_size(synth):
    t, _, _ = synth.workload("cfg2")
    assert_same_format(t.dims, t.inds, t.vals).close()


def test_errors():
    import torch

    dims = (50, 40, 30)
    rng = np.random.default_rng(1)
    inds, vals = _random(rng, dims, 500)
    bad = [i.copy() for i in inds]
    bad[1][7] = 40
    with pytest.raises(B.HbcsfError) as e:
        _device_tensor(dims, bad, vals)
    assert e.value.code == -2
    with pytest.raises(B.HbcsfError) as e:
        B.device_build_bytes(dims, 10, fiber_threshold=5)
    assert e.value.code == -1
    with pytest.raises(B.HbcsfError) as e:                      # five 30-bit modes: a 150-bit key
        B.device_build_bytes((1 << 30,) * 5, 10)
    assert e.value.code == -2
    arena_bytes, ws_bytes = B.device_build_bytes(dims, len(vals))
    di = [torch.from_numpy(x.view(np.int32)).cuda() for x in inds]
    dv = torch.from_numpy(vals).cuda()
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ptrs = [x.data_ptr() for x in di]
    with pytest.raises(B.HbcsfError) as e:                      # arena too small for the arrays
        B.build_format_device(dims, len(vals), ptrs, dv.data_ptr(), arena.data_ptr(), 1024, ws.data_ptr(), ws_bytes)
    assert e.value.code == -3
    with pytest.raises(B.HbcsfError) as e:
        B.build_format_device(dims, len(vals), ptrs, dv.data_ptr(), arena.data_ptr(), arena_bytes, ws.data_ptr(), 4096)
    assert e.value.code == -3
    h = B.build_format_device(dims, len(vals), ptrs, dv.data_ptr(), arena.data_ptr(), arena_bytes, ws.data_ptr(), ws_bytes)
    with pytest.raises(B.HbcsfError) as e:                      # already resident
        B.upload(h, arena.data_ptr(), arena_bytes)
    assert e.value.code == -4
    B.free(h)
