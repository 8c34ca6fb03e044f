"""Randomised CPU check of the builder: for arbitrary small tensors (duplicates, empty slices, any
option) the emulated kernel schedule over the built arrays equals the oracle, every row is defined
exactly once, and the arrays expand back to the input."""
import numpy as np
from hypothesis import given, settings, strategies as st, HealthCheck

import format_walk as FW
from paper_1904_03329_amd import binding as B


@st.composite
def tensors(draw):
    order = draw(st.sampled_from([3, 4, 5]))
    dims = tuple(draw(st.integers(1, 12 if order < 5 else 6)) for _ in range(order))
    nnz = draw(st.integers(0, 300))
    seed = draw(st.integers(0, 2**31 - 1))
    skew = draw(st.booleans())
    rng = np.random.default_rng(seed)
    inds = []
    for d in dims:
        if skew:
            w = 1.0 / np.arange(1, d + 1) ** 1.5
            inds.append(rng.choice(d, size=nnz, p=w / w.sum()).astype(np.uint32))
        else:
            inds.append(rng.integers(0, d, size=nnz).astype(np.uint32))
    vals = rng.uniform(-1, 1, size=nnz).astype(np.float32)
    opts = dict(fiber_threshold=draw(st.sampled_from([0, 8, 16, 32, 64])),
                group_mask=draw(st.integers(0, 4)), mode_order_policy=draw(st.integers(0, 2)),
                hybrid_granularity=draw(st.integers(0, 1)), coo_row_flags=draw(st.integers(0, 1)),
                mid_blocking=draw(st.sampled_from([0, 1, 2, 3])))
    rank = draw(st.sampled_from([8, 16]))
    upw = draw(st.integers(1, 3))
    return dims, inds, vals, opts, rank, upw, seed


@settings(max_examples=200, deadline=None, suppress_health_check=[HealthCheck.too_slow, HealthCheck.function_scoped_fixture])
@given(tensors())
def test_any_small_tensor(oracle, case):
    dims, inds, vals, opts, rank, upw, seed = case
    rng = np.random.default_rng(seed + 1)
    facs = [rng.uniform(0, 1, size=(d, rank)).astype(np.float32) for d in dims]
    order = len(dims)
    h = B.build_format(dims, inds, vals, **opts)
    try:
        for mode in range(order):
            fmt = FW.read_mode(h, mode, order)
            st_ = fmt["stats"]
            assert sum(st_["group_nnz"]) == vals.shape[0]
            got = FW.emulate_kernels(fmt, facs, dims[mode], rank, units_per_wave=upw)
            want = oracle.mttkrp(dims, inds, vals, facs, mode)
            np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
            cols, v = FW.expand_to_coo(fmt)
            lm = fmt["level_mode"]
            a = np.stack([cols[lm.index(m)].astype(np.int64) for m in range(order)] + [v.view(np.uint32).astype(np.int64)])
            b = np.stack([x.astype(np.int64) for x in inds] + [vals.view(np.uint32).astype(np.int64)])
            assert np.array_equal(a[:, np.lexsort(a[::-1])], b[:, np.lexsort(b[::-1])])
            # COO row tables agree with the COO group
            bits = B.host_array(h, mode, 0, 0, B.ARR_COO_BITS)
            ptr = B.host_array(h, mode, 0, 0, B.ARR_COO_PTR)
            rows = [r for r in range(dims[mode]) if (bits[r >> 5] >> (r & 31)) & 1]
            assert rows == fmt["coo"]["ind"][0][: fmt["coo"]["nnz"]].tolist()
            assert ptr[-1] == fmt["coo"]["nnz"] and np.all(np.diff(ptr.astype(np.int64)) >= 0)
    finally:
        B.free(h)
