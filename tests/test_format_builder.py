"""Host format builder (no GPU): groups, splitting, run tables, storage counts, and two CPU walks
of the built arrays against the oracle."""
import os

import numpy as np
import pytest

import format_walk as FW
from paper_1904_03329_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _coo(rng, dims, nnz, unique=True):
    total = int(np.prod(dims))
    lin = rng.choice(total, size=min(nnz, total), replace=False) if unique else rng.integers(0, total, size=nnz)
    inds = [np.asarray(x, dtype=np.uint32) for x in np.unravel_index(lin, dims)]
    return inds, rng.uniform(-1, 1, size=lin.shape[0]).astype(np.float32)


def _skewed(rng, dims, nnz):
    """Power-law-ish coordinates so that heavy slices, heavy fibers and singletons all occur."""
    inds = []
    for d in dims:
        w = 1.0 / np.arange(1, d + 1) ** 1.3
        inds.append(rng.choice(d, size=nnz, p=w / w.sum()).astype(np.uint32))
    key = np.zeros(nnz, dtype=np.int64)
    for d, x in zip(dims, inds):
        key = key * d + x
    _, first = np.unique(key, return_index=True)
    inds = [x[first] for x in inds]
    return inds, rng.uniform(-1, 1, size=first.shape[0]).astype(np.float32)


def _factors(rng, dims, rank):
    return [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]


def test_storage_example_of_section_v():
    want = {}
    for line in open(os.path.join(GOLDEN, "storage_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            want[k] = int(v)
    # slice 0: one nonzero; slice 1: three single-nonzero fibers; slice 2: one fiber of four
    i = np.array([0, 1, 1, 1, 2, 2, 2, 2], np.uint32)
    j = np.array([3, 0, 1, 2, 1, 1, 1, 1], np.uint32)
    k = np.array([2, 0, 1, 2, 0, 1, 2, 3], np.uint32)
    v = np.arange(1, 9, dtype=np.float32)
    h = B.build_format((3, 4, 4), [i, j, k], v, mode_order_policy=2)
    st = B.get_stats(h, 0)
    assert st["slices"] == want["S"] and st["fibers"][0] == want["F"] and st["nnz"] == want["M"]
    assert st["words_coo"] == want["words_coo"]
    assert st["words_csf"] == want["words_csf"]
    assert st["words_hbcsf"] == want["words_hbcsf"]
    assert st["group_slices"] == [1, 1, 1] and st["group_nnz"] == [1, 3, 4]
    # third slice: CSF words 2 + 2*1 + 4 = 8 against COO's 3*4 = 12
    assert 3 * 4 - (2 + 2 * 1 + 4) == want["third_slice_saving"]
    B.free(h)


def test_storage_and_operation_closed_forms():
    rng = np.random.default_rng(1)
    dims = (60, 40, 30)
    inds, vals = _skewed(rng, dims, 5000)
    M = vals.shape[0]
    h = B.build_format(dims, inds, vals)
    for mode in range(3):
        st = B.get_stats(h, mode)
        S, F = st["slices"], st["fibers"][0]
        assert st["words_coo"] == 3 * M                       # Section III-A
        assert st["words_csf"] == 2 * S + 2 * F + M           # Section III-B
        assert M <= st["words_hbcsf"] <= 3 * M                # Section V: between 1M and 3M words
        assert st["words_hbcsf"] <= st["words_csf"]           # Section VI-F: never more than CSF
        assert 2 * M <= st["flops_real"] <= 4 * M             # Section III-B: 2MR .. 4MR
        assert sum(st["group_nnz"]) == M and sum(st["group_slices"]) == S
    B.free(h)


@pytest.mark.parametrize("dims,nnz", [((30, 20, 25), 1500), ((12, 9, 10, 7), 1200), ((40, 3, 500), 900),
                                      ((9, 6, 7, 5, 4), 1500)])
@pytest.mark.parametrize("tf", [8, 32])
def test_round_trip_and_structure(dims, nnz, tf):
    rng = np.random.default_rng(len(dims) * 100 + tf)
    inds, vals = _skewed(rng, dims, nnz)
    order = len(dims)
    h = B.build_format(dims, inds, vals, fiber_threshold=tf)
    for mode in range(order):
        fmt = FW.read_mode(h, mode, order)
        lm = fmt["level_mode"]
        assert lm[0] == mode and sorted(lm) == list(range(order))
        cols, v = FW.expand_to_coo(fmt)
        # the same multiset of (coordinates, value)
        got = np.stack([cols[lm.index(m)].astype(np.int64) for m in range(order)] + [v.view(np.uint32).astype(np.int64)])
        want = np.stack([x.astype(np.int64) for x in inds] + [vals.view(np.uint32).astype(np.int64)])
        assert np.array_equal(got[:, np.lexsort(got[::-1])], want[:, np.lexsort(want[::-1])])
        # group rules of Section V
        cnt = np.bincount(inds[mode], minlength=dims[mode])
        coo = fmt["coo"]
        assert np.all(cnt[coo["ind"][0][: coo["nnz"]]] == 1)
        csl = fmt["csl"]
        if csl["nnz"]:
            n = csl["slices"]
            lens = np.diff(csl["ptr"][0][: n + 1].astype(np.int64))
            assert np.all(lens > 1)
            for s in range(n):
                a, b = csl["ptr"][0][s], csl["ptr"][0][s + 1]
                mids = np.stack([csl["ind"][l][a:b] for l in range(1, order - 1)])
                assert np.unique(mids, axis=1).shape[1] == b - a      # every fiber a singleton
        csf = fmt["csf"]
        L = fmt["L"]
        assert L == tf
        if csf["nnz"]:
            for l in range(order - 1):
                n = len(csf["ind"][l]) - 1
                ptr = csf["ptr"][l].astype(np.int64)
                assert ptr[0] == 0 and ptr[n] == csf["nnz"] and np.all(np.diff(ptr) > 0)
                if l > 0:
                    assert np.all(np.diff(ptr) <= L)                    # fbr-split bound
                    assert np.all(ptr[:-1] // L == (ptr[1:] - 1) // L)   # no segment crosses a run
                    assert np.isin(ptr, csf["ptr"][l + 1].astype(np.int64)).all() if l + 1 < order - 1 else True
                run = csf["run"][l].astype(np.int64)
                runs = (csf["nnz"] + L - 1) // L
                assert run.shape[0] == runs + 1 and run[runs] == n
                for r in range(runs):
                    assert ptr[run[r]] <= r * L < ptr[run[r] + 1]
            # every slice of the CSF group has a fiber with two or more nonzeros
            n0 = len(csf["ind"][0]) - 1
            own = (csf["ind"][0][:n0] & B.OWNED_BIT) != 0
            p0 = csf["ptr"][0].astype(np.int64)
            assert np.array_equal(own, p0[:-1] // L == (p0[1:] - 1) // L)
        # owned bitmap = COO rows + slices inside one run
        bits = fmt["owned"]
        owned_rows = {r for r in range(dims[mode]) if (bits[r >> 5] >> (r & 31)) & 1}
        exp = set(coo["ind"][0][: coo["nnz"]].tolist())
        for grp in (csl, csf):
            n0 = grp["slices"]
            if n0:
                ind0 = grp["ind"][0][:n0]
                exp |= set((ind0[(ind0 & B.OWNED_BIT) != 0] & 0x7FFFFFFF).tolist())
        assert owned_rows == exp
        assert fmt["stats"]["owned_rows"] == len(exp)
    B.free(h)


@pytest.mark.parametrize("dims,nnz,rank", [((30, 20, 25), 1500, 8), ((12, 9, 10, 7), 1200, 8), ((5, 400, 6), 1000, 32),
                                           ((9, 8, 7, 6), 700, 32), ((8, 6, 7, 5, 4), 1500, 8), ((6, 5, 4, 3, 50), 900, 32)])
@pytest.mark.parametrize("opts", [dict(), dict(fiber_threshold=8), dict(group_mask=4), dict(group_mask=1),
                                  dict(group_mask=2, mode_order_policy=1)])
def test_cpu_walks_match_oracle(oracle, dims, nnz, rank, opts):
    rng = np.random.default_rng(abs(hash((dims, rank, tuple(sorted(opts.items()))))) % 2**32)
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors(rng, dims, rank)
    order = len(dims)
    h = B.build_format(dims, inds, vals, **opts)
    for mode in range(order):
        want = oracle.mttkrp(dims, inds, vals, facs, mode)
        fmt = FW.read_mode(h, mode, order)
        if opts.get("group_mask") == 4:
            assert fmt["coo"]["nnz"] == 0 and fmt["csl"]["nnz"] == 0
        got = FW.walk_algorithms(fmt, facs, dims[mode], rank)
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
        for upw in (1, 3):
            got = FW.emulate_kernels(fmt, facs, dims[mode], rank, units_per_wave=upw)
            np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)
    B.free(h)


def test_uniform_small_workload_cfg1(oracle, synth):
    t, facs, rank = synth.workload("cfg1")
    h = B.build_format(t.dims, t.inds, t.vals)
    for mode in range(3):
        fmt = FW.read_mode(h, mode, 3)
        got = FW.emulate_kernels(fmt, facs, t.dims[mode], rank)
        np.testing.assert_allclose(got, oracle.mttkrp(t.dims, t.inds, t.vals, facs, mode), rtol=1e-11, atol=1e-12)
    B.free(h)


def test_split_arithmetic_examples():
    """Section VI-B's example: a fiber of 32 nonzeros with threshold 16 becomes 2 segments; Section
    IV-A's: a slice of 2048 nonzeros with 512 per worker is shared by 4 workers."""
    i = np.zeros(32, np.uint32)
    j = np.zeros(32, np.uint32)
    k = np.arange(32, dtype=np.uint32)
    h = B.build_format((1, 1, 32), [i, j, k], np.ones(32, np.float32), fiber_threshold=16, mode_order_policy=2)
    st = B.get_stats(h, 0)
    assert st["fibers"][0] == 1 and st["segments"][0] == 2 and st["runs"][2] == 2
    B.free(h)
    n = 2048
    h = B.build_format((1, 64, 32), [np.zeros(n, np.uint32), (np.arange(n) // 32).astype(np.uint32),
                                     (np.arange(n) % 32).astype(np.uint32)], np.ones(n, np.float32),
                       fiber_threshold=32, mode_order_policy=2)
    st = B.get_stats(h, 0)
    lane_groups, L = 8, 32                      # rank 32: 8 lane groups per wavefront
    units = -(-st["runs"][2] // lane_groups)
    ts = 512
    waves = -(-units // (ts // (lane_groups * L)))
    assert waves == 4 and st["shared_slices"] == 1
    B.free(h)


def test_duplicates_empty_and_errors(oracle):
    rng = np.random.default_rng(3)
    dims = (6, 5, 4)
    inds, vals = _coo(rng, dims, 200, unique=False)       # many duplicate coordinates
    facs = _factors(rng, dims, 8)
    h = B.build_format(dims, inds, vals)
    for mode in range(3):
        fmt = FW.read_mode(h, mode, 3)
        np.testing.assert_allclose(FW.emulate_kernels(fmt, facs, dims[mode], 8),
                                   oracle.mttkrp(dims, inds, vals, facs, mode), rtol=1e-11, atol=1e-12)
    B.free(h)
    # empty tensor
    h = B.build_format(dims, [np.zeros(0, np.uint32)] * 3, np.zeros(0, np.float32))
    st = B.get_stats(h, 1)
    assert st["nnz"] == 0 and st["slices"] == 0 and st["owned_rows"] == 0
    assert B.device_bytes(h) > 0
    B.free(h)
    # error paths forced from the host
    with pytest.raises(B.HbcsfError) as e:
        B.build_format((6, 5), [inds[0], inds[1]], vals)
    assert e.value.code == -1
    bad = [x.copy() for x in inds]
    bad[2][7] = 4
    with pytest.raises(B.HbcsfError) as e:
        B.build_format(dims, bad, vals)
    assert e.value.code == -2 and "dimension" in str(e.value)
    with pytest.raises(B.HbcsfError):
        B.build_format(dims, inds, vals, fiber_threshold=12)
    with pytest.raises(B.HbcsfError):
        B.build_format((2**31, 5, 4), inds, vals)
    h = B.build_format(dims, inds, vals)
    with pytest.raises(B.HbcsfError) as e:      # mttkrp before upload
        B.mttkrp(h, 0, 8, [0, 1024, 2048], 4096)
    assert e.value.code == -4
    with pytest.raises(B.HbcsfError) as e:
        B.mttkrp(h, 0, 7, [0, 1024, 2048], 4096)
    assert e.value.code == -1
    with pytest.raises(B.HbcsfError):
        B.mttkrp(h, 3, 8, [0, 1024, 2048], 4096)
    with pytest.raises(B.HbcsfError):
        B.get_stats(h, -1)
    B.free(h)
    assert B.strerror(-2) == "index or size out of range"


def test_tuning_keys_are_validated():
    h = B.build_format((4, 4, 4), [np.array([1], np.uint32)] * 3, np.array([1.0], np.float32))
    B.tune(h, B.TUNE_SLICE_THRESHOLD, 4096)
    B.tune(h, B.TUNE_WAVES_PER_CU, 64)
    B.tune(h, B.TUNE_STEPS, 4)
    B.tune(h, B.TUNE_KERNEL_MASK, 8)
    B.tune(h, B.TUNE_PERSISTENT, 1)
    B.tune(h, B.TUNE_STREAM_BYTES, 0)
    B.tune(h, B.TUNE_TRACE_CAPACITY, 10)
    B.tune(h, B.TUNE_TRACE_BUFFER, 0)
    for key, bad in ((B.TUNE_STEPS, 5), (B.TUNE_KERNEL_MASK, 16), (B.TUNE_WAVES_PER_CU, 5000),
                     (B.TUNE_TRACE_BUFFER, 12), (99, 1)):
        with pytest.raises(B.HbcsfError) as e:
            B.tune(h, key, bad)
        assert e.value.code == -1
    with pytest.raises(B.HbcsfError) as e:       # no profiled call yet
        B.kernel_ms(h, 0)
    assert e.value.code == -4
    B.free(h)


def test_wide_coordinates_use_the_128_bit_sort_key(oracle):
    """Dimensions whose packed coordinate exceeds 64 bits (as FROSTT's larger tensors do)."""
    rng = np.random.default_rng(5)
    dims = (2**30, 2**29 + 3, 2**28)
    n = 3000
    inds = [rng.integers(0, 50, size=n).astype(np.uint32) * np.uint32(d // 64) for d in dims]
    vals = rng.uniform(-1, 1, size=n).astype(np.float32)
    h = B.build_format(dims, inds, vals)
    for mode in range(3):
        fmt = FW.read_mode(h, mode, 3)
        cols, v = FW.expand_to_coo(fmt)
        lm = fmt["level_mode"]
        got = np.stack([cols[lm.index(m)].astype(np.int64) for m in range(3)] + [v.view(np.uint32).astype(np.int64)])
        want = np.stack([x.astype(np.int64) for x in inds] + [vals.view(np.uint32).astype(np.int64)])
        assert np.array_equal(got[:, np.lexsort(got[::-1])], want[:, np.lexsort(want[::-1])])
    B.free(h)


def test_library_exports_every_declared_symbol():
    import ctypes
    import re
    header = open(os.path.join(os.path.dirname(GOLDEN), "..", "include", "hbcsf.h")).read()
    declared = set(re.findall(r"\b(hbcsf_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("order", [3, 4])
def test_per_fiber_hybrid_splits_heavy_slices(oracle, order):
    """hybrid_granularity = 1 (Section VI-F's open point): inside a slice of at least 2 T_f nonzeros the nonzeros of
    singleton deepest-level fibers go to the CSL group and the others to the CSF group, as two pieces with the same
    root index, both merged with atomic adds; light slices and slices with few singleton fibers stay whole."""
    rng = np.random.default_rng(5 + order)
    L = 8
    dims = (6, 40, 50) if order == 3 else (6, 4, 40, 50)
    rows = []

    def add(root, mids, leaves):          # nonzeros (root, [mid...], leaf)
        for m, l in zip(mids, leaves):
            rows.append((root,) + tuple(m) + (l,))

    mid = (lambda j: (j,)) if order == 3 else (lambda j: (1, j))
    # slice 0: 30 nonzeros, 20 in singleton fibers + one fiber of 10 -> split
    add(0, [mid(j) for j in range(20)] + [mid(30)] * 10, list(range(20)) + list(range(10)))
    # slice 1: 30 nonzeros, 2 singleton fibers + 4 fibers of 7 -> too few singletons: stays in the CSF group
    add(1, [mid(0), mid(1)] + [mid(5 + q) for q in range(4) for _ in range(7)], [0, 1] + [r for _ in range(4) for r in range(7)])
    # slice 2: 10 nonzeros (below 2 T_f), 6 singleton fibers + one of 4 -> stays in the CSF group
    add(2, [mid(j) for j in range(6)] + [mid(9)] * 4, list(range(6)) + list(range(4)))
    # slice 3: all singleton fibers -> CSL as a whole; slice 4: one nonzero -> COO
    add(3, [mid(j) for j in range(20)], list(range(20)))
    add(4, [mid(3)], [3])
    arr = np.array(rows, dtype=np.uint32)
    arr = arr[rng.permutation(arr.shape[0])]
    inds = [np.ascontiguousarray(arr[:, m]) for m in range(order)]
    vals = rng.uniform(-1, 1, size=arr.shape[0]).astype(np.float32)
    facs = [rng.uniform(0, 1, size=(d, 8)).astype(np.float32) for d in dims]
    h = B.build_format(dims, inds, vals, fiber_threshold=L, mode_order_policy=2, hybrid_granularity=1)
    h0 = B.build_format(dims, inds, vals, fiber_threshold=L, mode_order_policy=2)
    try:
        st, st0 = B.get_stats(h, 0), B.get_stats(h0, 0)
        assert st0["group_nnz"] == [1, 20, 70] and st0["group_slices"] == [1, 1, 3]
        assert st["group_nnz"] == [1, 40, 50] and st["group_slices"] == [1, 2, 3]
        fmt = FW.read_mode(h, 0, order)
        csl_roots = (fmt["csl"]["ind"][0][:2] & 0x7FFFFFFF).tolist()
        csl_owned = (fmt["csl"]["ind"][0][:2] >> 31).tolist()
        csf_roots = (fmt["csf"]["ind"][0][:3] & 0x7FFFFFFF).tolist()
        csf_owned = (fmt["csf"]["ind"][0][:3] >> 31).tolist()
        assert csl_roots == [0, 3] and csf_roots == [0, 1, 2]
        assert csl_owned[0] == 0 and csf_owned[0] == 0            # both pieces of the split slice are shared
        assert not (fmt["owned"][0] & 1)                           # so its row is zero-filled, not stored
        # the CSL piece of slice 0 holds exactly the 20 singleton-fiber nonzeros
        ptr = fmt["csl"]["ptr"][0]
        assert ptr[1] - ptr[0] == 20
        assert sorted(fmt["csl"]["ind"][order - 2][ptr[0]:ptr[1]].tolist()) == list(range(20))
        # the CSF piece keeps the fiber of 10, cut on the run grid
        assert st["segments"][order - 3] >= 1 + 6 + 2
        for mode in range(order):
            f = FW.read_mode(h, mode, order)
            want = oracle.mttkrp(dims, inds, vals, facs, mode)
            np.testing.assert_allclose(FW.walk_algorithms(f, facs, dims[mode], 8), want, rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(FW.emulate_kernels(f, facs, dims[mode], 8), want, rtol=1e-10, atol=1e-12)
        with pytest.raises(B.HbcsfError):
            B.build_format(dims, inds, vals, hybrid_granularity=2)
    finally:
        B.free(h)
        B.free(h0)


@pytest.mark.parametrize("dims,nnz", [((6, 200, 300), 4000), ((5, 64, 9, 40), 3000), ((4, 33, 5, 3, 20), 2000)])
def test_level_one_blocking(oracle, dims, nnz):
    """mid_blocking (Section VIII: blocking as complementary work): with 2^b blocks over the level-1 index range the
    stream is ordered by (block, root, level 1, ..): every slice is stored as one piece per block it has nonzeros in,
    no piece owns its row, the COO group is unused, and the result is unchanged."""
    rng = np.random.default_rng(len(dims) * 7 + nnz)
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors(rng, dims, 8)
    order = len(dims)
    h = B.build_format(dims, inds, vals, fiber_threshold=8, mode_order_policy=2, mid_blocking=3)
    h0 = B.build_format(dims, inds, vals, fiber_threshold=8, mode_order_policy=2, mid_blocking=1)
    try:
        st, st0 = B.get_stats(h, 0), B.get_stats(h0, 0)
        fmt = FW.read_mode(h, 0, order)
        l1 = fmt["level_mode"][1]
        drop = max(int(np.ceil(np.log2(dims[l1]))), 1) - 3
        pieces = np.unique(np.stack([inds[0].astype(np.int64), inds[l1].astype(np.int64) >> drop]), axis=1).shape[1]
        assert st["slices"] == pieces and st0["slices"] == np.unique(inds[0]).shape[0]
        assert st["group_nnz"][0] == 0 and st["owned_rows"] == 0 and not fmt["owned"].any()
        assert st["fibers"][0] == st0["fibers"][0]                       # a block boundary never cuts a fiber
        # pieces are ordered by (block, root): roots restart from the smallest in every block
        for g in ("csl", "csf"):
            n = fmt[g]["slices"]
            assert not (fmt[g]["ind"][0][:n] >> 31).any()                # no piece is marked owned
        for mode in range(order):
            f = FW.read_mode(h, mode, order)
            want = oracle.mttkrp(dims, inds, vals, facs, mode)
            np.testing.assert_allclose(FW.walk_algorithms(f, facs, dims[mode], 8), want, rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(FW.emulate_kernels(f, facs, dims[mode], 8), want, rtol=1e-10, atol=1e-12)
        with pytest.raises(B.HbcsfError):
            B.build_format(dims, inds, vals, mid_blocking=14)
    finally:
        B.free(h)
        B.free(h0)


@pytest.mark.parametrize("dims,nnz", [((30, 20, 25), 1500), ((12, 9, 10, 7), 1200), ((6, 5, 7, 4, 9), 1500)])
def test_single_representation(oracle, dims, nnz):
    """single_representation = 1 (the one-representation setting Section VI-A sets aside for ALLMODE): only mode 0's
    plain B-CSF tree is stored; the walk that serves another mode -- start marks, target at a lower tree level, one
    atomic contribution per level-T segment -- reproduces the oracle for every mode."""
    rng = np.random.default_rng(len(dims) * 13 + nnz)
    inds, vals = _skewed(rng, dims, nnz)
    facs = _factors(rng, dims, 8)
    order = len(dims)
    h = B.build_format(dims, inds, vals, single_representation=1)
    h_all = B.build_format(dims, inds, vals, group_mask=4)
    try:
        assert B.device_bytes(h) == pytest.approx(B.device_bytes(h_all) / order, rel=0.5)
        assert B.device_bytes(h) < 0.6 * B.device_bytes(h_all)
        st = B.get_stats(h, 0)
        assert st["group_nnz"] == [0, 0, vals.shape[0]]
        with pytest.raises(B.HbcsfError) as e:
            B.get_stats(h, 1)
        assert e.value.code == -4
        fmt = FW.read_mode(h, 0, order)
        np.testing.assert_allclose(FW.emulate_kernels(fmt, facs, dims[0], 8), oracle.mttkrp(dims, inds, vals, facs, 0),
                                   rtol=1e-10, atol=1e-12)
        for mode in range(1, order):
            np.testing.assert_allclose(FW.emulate_nonroot(fmt, facs, mode, dims[mode], 8),
                                       oracle.mttkrp(dims, inds, vals, facs, mode), rtol=1e-10, atol=1e-12)
        for bad in (dict(group_mask=1), dict(fiber_threshold=8), dict(coo_row_flags=1), dict(mid_blocking=3)):
            with pytest.raises(B.HbcsfError):
                B.build_format(dims, inds, vals, single_representation=1, **bad)
    finally:
        B.free(h)
        B.free(h_all)
