"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same inputs."""
import numpy as np
import pytest

import gpu_util as GU
from paper_1904_03329_amd import binding as B

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


def _factors(rng, dims, rank):
    return [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]


def _check_all_modes(oracle, dims, inds, vals, facs, what, **kw):
    outs, stats = GU.gpu_mttkrp_all_modes(dims, inds, vals, facs, **kw)
    for mode, got in enumerate(outs):
        want = oracle.mttkrp(dims, inds, vals, facs, mode)
        GU.assert_close(got, want, f"{what} mode {mode}")
    return stats


def test_cfg1_every_element(oracle, synth):
    t, facs, rank = synth.workload("cfg1")
    print("cfg1", t.dims, t.nnz, rank, flush=True)
    _check_all_modes(oracle, t.dims, t.inds, t.vals, facs, "cfg1")


@pytest.mark.parametrize("rank", [8, 16, 32, 64, 128])
@pytest.mark.parametrize("dims,nnz", [((3000, 700, 90), 60_000), ((900, 300, 40, 25), 50_000),
                                      ((600, 200, 30, 12, 8), 50_000)])
def test_ranks_and_orders(oracle, dims, nnz, rank):
    rng = np.random.default_rng(rank * 10 + len(dims))
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors(rng, dims, rank)
    print("ranks_and_orders", dims, vals.shape[0], rank, flush=True)
    stats = _check_all_modes(oracle, dims, inds, vals, facs, f"R={rank} order={len(dims)}")
    assert all(s["group_nnz"][2] > 0 for s in stats)


@pytest.mark.parametrize("opts", [dict(fiber_threshold=8), dict(fiber_threshold=64), dict(group_mask=4),
                                  dict(group_mask=1), dict(group_mask=2), dict(mode_order_policy=1),
                                  dict(mode_order_policy=2), dict(tune_ts=256), dict(tune_ts=100_000),
                                  dict(hybrid_granularity=1), dict(hybrid_granularity=1, fiber_threshold=8),
                                  dict(coo_row_flags=1), dict(mid_blocking=4), dict(mid_blocking=2, fiber_threshold=8),
                                  dict(tune_dense=1),
                                  dict(tune_dense=1, fiber_threshold=32), dict(tune_dense=1, group_mask=4, tune_ts=256),
                                  dict(tune_dense=1, tune_steps=4)])
@pytest.mark.parametrize("dims,nnz", [((5000, 400, 60), 120_000), ((2000, 100, 30, 12), 90_000),
                                      ((1500, 80, 20, 9, 6), 90_000)])
def test_build_options_do_not_change_the_result(oracle, dims, nnz, opts):
    rng = np.random.default_rng(len(dims) + 7)
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors(rng, dims, 32)
    print("options", dims, vals.shape[0], opts, flush=True)
    _check_all_modes(oracle, dims, inds, vals, facs, f"{opts}", **opts)


def test_hypersparse_groups(oracle, synth):
    """Long-tail tensor: most slices hold one or two nonzeros, so the COO and CSL groups carry work."""
    t = synth.tensor((400_000, 400_000, 100), 600_000, (1.05, 1.05, 0.0), seed=77)
    facs = synth.factors(t.dims, 32, seed=77)
    print("hypersparse", t.dims, t.nnz, flush=True)
    stats = _check_all_modes(oracle, t.dims, t.inds, t.vals, facs, "hypersparse")
    assert stats[0]["group_nnz"][0] > 0 and stats[0]["group_nnz"][1] > 0 and stats[0]["group_nnz"][2] > 0
    # the per-fiber choice moves the singleton-fiber nonzeros of heavy slices from the CSF to the CSL group
    split = _check_all_modes(oracle, t.dims, t.inds, t.vals, facs, "hypersparse, per-fiber groups", hybrid_granularity=1)
    assert split[0]["group_nnz"][1] > stats[0]["group_nnz"][1] and split[0]["group_nnz"][0] == stats[0]["group_nnz"][0]
    # COO group without stored root indices (row flags): one index word less per nonzero, same result
    flags = _check_all_modes(oracle, t.dims, t.inds, t.vals, facs, "hypersparse, COO row flags", coo_row_flags=1)
    assert flags[0]["stream_bytes"][0] < stats[0]["stream_bytes"][0] and flags[0]["group_nnz"] == stats[0]["group_nnz"]


@pytest.mark.parametrize("dims,nnz,alpha", [((34_000_000, 34_000_000, 100), 1_500_000, (1.05, 1.05, 0.0)),
                                            ((34_000_000, 3000, 60, 20), 1_000_000, (1.05, 1.1, 1.0, 0.8))])
def test_factor_matrices_above_4GiB(oracle, synth, dims, nnz, alpha):
    """Factor matrices of 34 M rows x 32 floats exceed 4 GiB, so every kernel runs in its 64-bit-offset
    instantiation (orders 3 and 4).  Every non-empty output row is compared with the oracle and every other
    row must be exactly zero."""
    import torch
    from paper_1904_03329_amd import HbcsfTensor

    with open("/proc/meminfo") as f:
        avail = [int(l.split()[1]) for l in f if l.startswith("MemAvailable:")][0] / (1 << 20)
    if avail < 24:
        pytest.skip(f"needs about 24 GiB of host memory for the factor matrices, {avail:.0f} GiB available")
    t = synth.tensor(dims, nnz, alpha, seed=4242)
    facs = synth.factors(t.dims, 32, seed=4242)
    print("wide", t.dims, t.nnz, flush=True)
    ht = HbcsfTensor(t.dims, t.inds, t.vals).to_device()
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    for mode in range(t.order):
        st = ht.stats(mode)
        out = torch.full((t.dims[mode], 32), float("nan"), dtype=torch.float32, device="cuda")
        ht.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        rows = np.unique(t.inds[mode])
        want = oracle.mttkrp_rows(t.dims, t.inds, t.vals, facs, mode, rows)
        drows = torch.from_numpy(rows.astype(np.int64)).cuda()
        rel = GU.assert_close(out[drows].cpu().numpy(), want, f"wide order {t.order} mode {mode}")
        out[drows] = 0.0
        assert int(torch.count_nonzero(out)) == 0 and bool(torch.isfinite(out).all()), "an empty slice's row is not zero"
        print(f"wide order {t.order} mode {mode}: {rows.size} non-empty rows, groups {st['group_nnz']}, "
              f"max|diff|/max|M| = {rel:.2e}", flush=True)
        del out
    ht.close()


@pytest.mark.parametrize("dims,nnz,a", [((2000, 30, 4000), 300_000, 0.4), ((300, 3, 12, 3000), 250_000, 0.3),
                                        ((50_000, 20_000, 300), 400_000, 1.2)])
def test_dense_fiber_row_gather(oracle, dims, nnz, a):
    """The B-CSF kernel's dense gather of fiber-level rows (HBCSF_TUNE_DENSE_MID = 1) on long fibers (few marks per
    block of steps), on a 4-order tensor (two fiber levels share the row cache) and on a tensor whose fibers are
    mostly singletons, so that a block's marks overflow the 32-row cache and take the direct-load path."""
    rng = np.random.default_rng(len(dims) * 31 + nnz % 97)
    inds, vals = _skewed(rng, dims, nnz, a=a)
    facs = _factors(rng, dims, 32)
    print("dense gather", dims, vals.shape[0], flush=True)
    for mask in (0, 4):
        stats = _check_all_modes(oracle, dims, inds, vals, facs, f"dense gather mask {mask}", tune_dense=1, group_mask=mask)
    assert all(s["group_nnz"][2] == vals.shape[0] for s in stats)


@pytest.mark.parametrize("dims,nnz,a", [((3000, 700, 90), 200_000, 1.3), ((900, 300, 40, 25), 150_000, 1.2),
                                        ((600, 200, 30, 12, 8), 120_000, 1.1), ((40, 9000, 11_000), 90_000, 0.6),
                                        ((3, 50, 4000), 10_007, 0.0)])
def test_single_representation(oracle, dims, nnz, a):
    """single_representation = 1: mode 0 from its own B-CSF tree, every other mode from the same tree with the
    target at a lower level (atomic contributions), rank 32; heavy slices, long fibers, a ragged last unit."""
    import torch
    from paper_1904_03329_amd import HbcsfTensor

    rng = np.random.default_rng(len(dims) * 17 + nnz % 89)
    if a > 0:
        inds, vals = _skewed(rng, dims, nnz, a=a)
    else:
        inds = [rng.integers(0, d, nnz).astype(np.uint32) for d in dims]
        vals = rng.uniform(-1, 1, nnz).astype(np.float32)
    facs = _factors(rng, dims, 32)
    print("single representation", dims, vals.shape[0], flush=True)
    t = HbcsfTensor(dims, inds, vals, single_representation=1).to_device()
    full = HbcsfTensor(dims, inds, vals, group_mask=4)
    assert B.device_bytes(t.handle) < 0.6 * B.device_bytes(full.handle)
    full.close()
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    for mode in range(len(dims)):
        out = torch.full((dims[mode], 32), float("nan"), dtype=torch.float32, device="cuda")
        t.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), oracle.mttkrp(dims, inds, vals, facs, mode), f"single representation mode {mode}")
    f8 = [torch.zeros((d, 8), device="cuda") for d in dims]
    with pytest.raises(B.HbcsfError) as e:
        t.mttkrp(1, f8, torch.zeros((dims[1], 8), device="cuda"))
    assert e.value.code == -1
    t.close()


def test_degenerate_shapes(oracle):
    rng = np.random.default_rng(31)
    # one heavy slice only (every partial row merged with atomics), ragged tail
    n = 10_007
    dims = (3, 50, 4000)
    inds = [np.full(n, 1, np.uint32), rng.integers(0, 50, n).astype(np.uint32), rng.integers(0, 4000, n).astype(np.uint32)]
    vals = rng.uniform(-1, 1, n).astype(np.float32)
    facs = _factors(rng, dims, 32)
    print("one heavy slice", flush=True)
    _check_all_modes(oracle, dims, inds, vals, facs, "one heavy slice")
    # every slice a single nonzero (COO group only) and empty rows in between
    dims = (5000, 7, 9)
    rows = rng.permutation(5000)[:1234].astype(np.uint32)
    inds = [rows, rng.integers(0, 7, 1234).astype(np.uint32), rng.integers(0, 9, 1234).astype(np.uint32)]
    vals = rng.uniform(-1, 1, 1234).astype(np.float32)
    facs = _factors(rng, dims, 8)
    print("singleton slices", flush=True)
    stats = _check_all_modes(oracle, dims, inds, vals, facs, "singleton slices")
    assert stats[0]["group_nnz"] == [1234, 0, 0]
    # a single nonzero; and an empty tensor (the result must be all zeros, not stale memory)
    print("single nonzero / empty", flush=True)
    _check_all_modes(oracle, (4, 5, 6), [np.array([3], np.uint32), np.array([0], np.uint32), np.array([5], np.uint32)],
                     np.array([0.5], np.float32), _factors(rng, (4, 5, 6), 16), "single nonzero")
    outs, _ = GU.gpu_mttkrp_all_modes((40, 5, 6, 3), [np.zeros(0, np.uint32)] * 4, np.zeros(0, np.float32),
                                      _factors(rng, (40, 5, 6, 3), 32))
    assert all(np.array_equal(o, np.zeros_like(o)) for o in outs)
    # duplicate coordinates act as separate nonzeros
    dims = (30, 20, 10)
    inds = [rng.integers(0, d, 5000).astype(np.uint32) for d in dims]
    vals = rng.uniform(-1, 1, 5000).astype(np.float32)
    print("duplicates", flush=True)
    _check_all_modes(oracle, dims, inds, vals, _factors(rng, dims, 32), "duplicates")


def test_nan_and_inf_propagate_to_their_rows_only(oracle):
    rng = np.random.default_rng(37)
    dims = (200, 30, 20)
    inds, vals = _skewed(rng, dims, 4000)
    vals = vals.copy()
    vals[10] = np.nan
    vals[20] = np.inf
    facs = _factors(rng, dims, 32)
    import torch
    from paper_1904_03329_amd import HbcsfTensor
    t = HbcsfTensor(dims, inds, vals).to_device()
    out = t.mttkrp(0, [torch.from_numpy(f).cuda() for f in facs]).cpu().numpy()
    bad_rows = {int(inds[0][10]), int(inds[0][20])}
    for r in range(dims[0]):
        assert np.all(np.isfinite(out[r])) == (r not in bad_rows)
    t.close()


def test_repeated_calls_overwrite(oracle):
    rng = np.random.default_rng(41)
    dims = (800, 90, 40)
    inds, vals = _skewed(rng, dims, 30_000)
    facs = _factors(rng, dims, 32)
    import torch
    from paper_1904_03329_amd import HbcsfTensor
    t = HbcsfTensor(dims, inds, vals).to_device()
    d = [torch.from_numpy(f).cuda() for f in facs]
    out = torch.full((dims[1], 32), 123.0, device="cuda")
    want = oracle.mttkrp(dims, inds, vals, facs, 1)
    for _ in range(3):
        t.mttkrp(1, d, out)
        torch.cuda.synchronize()
        GU.assert_close(out.cpu().numpy(), want, "repeat")
    # a side stream works too
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out2 = t.mttkrp(1, d)
    s.synchronize()
    GU.assert_close(out2.cpu().numpy(), want, "side stream")
    # profiling hooks report the four kernels
    B.tune(t.handle, B.TUNE_PROFILE, 4)
    for mode in (0, 1):
        t.mttkrp(mode, d)
    for back in (0, 1):
        ms = B.kernel_ms(t.handle, back)
        assert len(ms) == 4 and ms[0] > 0 and ms[3] > 0
    with pytest.raises(B.HbcsfError):
        B.kernel_ms(t.handle, 2)
    t.close()


def test_launch_variants_and_diagnostics(oracle):
    """Persistent span walk, streaming middle-level loads, 4 gathers in flight, the kernel mask, the
    wavefront trace and the row-gather probe."""
    import torch
    from paper_1904_03329_amd import HbcsfTensor
    rng = np.random.default_rng(43)
    dims = (6000, 500, 70)
    inds, vals = _skewed(rng, dims, 150_000)
    facs = _factors(rng, dims, 32)
    want = [oracle.mttkrp(dims, inds, vals, facs, m) for m in range(3)]
    t = HbcsfTensor(dims, inds, vals).to_device()
    d = [torch.from_numpy(f).cuda() for f in facs]
    for key, value in ((B.TUNE_PERSISTENT, 1), (B.TUNE_STREAM_BYTES, 1), (B.TUNE_STEPS, 4), (B.TUNE_WAVES_PER_CU, 7),
                       (B.TUNE_FUSE_COO, 0), (B.TUNE_FUSE_COO, 1)):
        B.tune(t.handle, key, value)
        for m in range(3):
            GU.assert_close(t.mttkrp(m, d).cpu().numpy(), want[m], f"tune {key}={value} mode {m}")
    # the four kernels one by one give the same result as one call
    out = torch.full((dims[0], 32), float("nan"), device="cuda")
    for mask in (1, 2, 4, 8):
        B.tune(t.handle, B.TUNE_KERNEL_MASK, mask)
        t.mttkrp(0, d, out)
    B.tune(t.handle, B.TUNE_KERNEL_MASK, 15)
    GU.assert_close(out.cpu().numpy(), want[0], "kernel by kernel")
    # trace: one record per wavefront of the CSL and B-CSF kernels, on at most 256 compute units
    cap = 1 << 16
    buf = torch.zeros(4 + 4 * cap, dtype=torch.int64, device="cuda")
    B.tune(t.handle, B.TUNE_TRACE_CAPACITY, cap)
    B.tune(t.handle, B.TUNE_TRACE_BUFFER, buf.data_ptr())
    GU.assert_close(t.mttkrp(0, d).cpu().numpy(), want[0], "traced call")
    n = int(buf[0].item())
    rec = buf[4:4 + 4 * n].cpu().numpy().reshape(n, 4)
    assert 0 < n <= cap and set(np.unique(rec[:, 0]).tolist()) <= {1, 2}
    assert np.all(rec[:, 3] >= rec[:, 2])
    cu = ((rec[:, 1] >> 32) << 8) | ((((rec[:, 1] & 0xFFFFFFFF) >> 8) & 0xFF))
    assert np.unique(cu).size <= 256
    B.tune(t.handle, B.TUNE_TRACE_BUFFER, 0)
    t.close()
    # the probe gathers what it says and rejects bad arguments
    idx = torch.randint(0, 1000, (1 << 17,), device="cuda").to(torch.int32)
    table = torch.ones((1000, 32), device="cuda")
    sink = torch.zeros(4, device="cuda")
    rows, instr = B.probe_row_gather(idx.data_ptr(), idx.numel(), table.data_ptr(), 1000, sink.data_ptr())
    torch.cuda.synchronize()
    assert 0 < rows <= idx.numel() and rows == 8 * instr
    rows2, instr2 = B.probe_row_gather(idx.data_ptr(), idx.numel(), table.data_ptr(), 1000, sink.data_ptr(), 0, 2)
    torch.cuda.synchronize()
    assert instr2 == instr and rows2 == 2 * instr
    with pytest.raises(B.HbcsfError):
        B.probe_row_gather(idx.data_ptr(), idx.numel(), table.data_ptr(), 1000, sink.data_ptr(), 0, 9)
    with pytest.raises(B.HbcsfError):
        B.probe_row_gather(idx.data_ptr(), 10, table.data_ptr(), 1000, sink.data_ptr())


@pytest.mark.parametrize("seed", range(16))
def test_random_small_tensors(oracle, seed):
    """Small random tensors with duplicates, empty slices and every option drawn at random."""
    rng = np.random.default_rng(1000 + seed)
    order = int(rng.choice([3, 4, 5]))
    dims = tuple(int(x) for x in rng.integers(1, 60 if order < 5 else 25, size=order))
    nnz = int(rng.integers(0, 6000))
    inds = [rng.integers(0, d, size=nnz).astype(np.uint32) for d in dims]
    vals = rng.uniform(-1, 1, size=nnz).astype(np.float32)
    rank = int(rng.choice([8, 16, 32, 64]))
    opts = dict(fiber_threshold=int(rng.choice([0, 8, 16, 32, 64])), group_mask=int(rng.integers(0, 5)),
                mode_order_policy=int(rng.integers(0, 3)))
    print("random", seed, dims, nnz, rank, opts, flush=True)
    _check_all_modes(oracle, dims, inds, vals, _factors(rng, dims, rank), f"random {seed}", **opts)


def test_calls_replay_from_a_hip_graph(oracle):
    """hbcsf_mttkrp only launches kernels on the caller's stream (the output is cleared by a fill kernel, not a
    memset), so a step over all modes can be captured once and replayed; every replay, with eager work and
    synchronisations in between, must reproduce the eager result."""
    import torch
    from paper_1904_03329_amd import HbcsfTensor

    rng = np.random.default_rng(4242)
    dims, rank = (4000, 500, 70), 32
    inds, vals = _skewed(rng, dims, 150_000)
    facs = _factors(rng, dims, rank)
    t = HbcsfTensor(dims, inds, vals).to_device()
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    outs = [torch.empty((d, rank), dtype=torch.float32, device="cuda") for d in dims]
    eager = []
    for mode in range(3):                       # also warms up the launch-size queries
        t.mttkrp(mode, dfacs, outs[mode])
    torch.cuda.synchronize()
    for mode in range(3):
        GU.assert_close(outs[mode].cpu().numpy(), oracle.mttkrp(dims, inds, vals, facs, mode), f"eager mode {mode}")
        eager.append(outs[mode].clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for mode in range(3):
                t.mttkrp(mode, dfacs, outs[mode])
    torch.cuda.synchronize()
    for replay in range(3):
        for o in outs:
            o.fill_(float("nan"))               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for mode in range(3):
            got, want = outs[mode], eager[mode]
            assert bool(torch.isfinite(got).all()), f"replay {replay} mode {mode}"
            # atomics may merge in another order: same tolerance as against the oracle
            assert float((got - want).abs().max()) <= GU.REL_TOL * float(want.abs().max())
    t.close()
