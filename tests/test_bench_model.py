"""The benchmark's algorithmic-byte model, recounted from the format arrays themselves (no GPU needed).

`bench.py` prices a mode at: every format array once, 4 * rank bytes per distinct factor row a kernel gathers, and
4 * rank bytes per output row (rows a group stores in the kernel of that group, every other row as zero fill).  The
recount below takes the arrays through `hbcsf_host_array` and numpy instead of the builder's statistics."""
import importlib.util
import os

import numpy as np
import pytest

from paper_1904_03329_amd import HbcsfTensor, binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _skewed(rng, dims, nnz, a=1.2):
    inds = []
    for d in dims:
        w = 1.0 / np.arange(1, d + 1) ** a
        inds.append(rng.permutation(d)[rng.choice(d, size=nnz, p=w / w.sum())].astype(np.uint32))
    key = np.zeros(nnz, dtype=np.int64)
    for d, x in zip(dims, inds):
        key = key * d + x
    _, first = np.unique(key, return_index=True)
    return [x[first] for x in inds], rng.uniform(-1, 1, size=first.shape[0]).astype(np.float32)


def _array(h, mode, g, lvl, aid):
    try:
        return B.host_array(h, mode, g, lvl, aid)
    except B.HbcsfError:
        return None


@pytest.mark.parametrize("dims,nnz,rank,elem", [((3000, 400, 60), 40_000, 32, 4), ((700, 90, 30, 12), 30_000, 16, 4),
                                                ((3000, 400, 60), 40_000, 32, 8)])
def test_algorithmic_bytes_recounted_from_the_arrays(dims, nnz, rank, elem):
    bench = _bench()
    rng = np.random.default_rng(len(dims) + rank + elem)
    inds, vals = _skewed(rng, dims, nnz)
    order = len(dims)
    t = HbcsfTensor(dims, inds, vals)
    row = elem * rank
    for mode in range(order):
        st = t.stats(mode)
        st["rows"] = dims[mode]
        got = bench.algorithmic_bytes(st, rank, order, elem)
        owned = B.host_array(t.handle, mode, 0, 0, B.ARR_OWNED_BITS)
        owned_rows = int(np.unpackbits(owned.view(np.uint8)).sum())
        want_total = 4 * ((dims[mode] + 31) // 32) + row * dims[mode]
        for g, name in enumerate(("coo", "csl", "csf")):
            val = _array(t.handle, mode, g, 0, B.ARR_VAL)
            if val is None or st["group_nnz"][g] == 0:
                assert got[name] == 0
                continue
            words, gathered = val.size, 0
            for lvl in range(order):
                ind = _array(t.handle, mode, g, lvl, B.ARR_IND)
                for aid in (B.ARR_IND, B.ARR_PTR, B.ARR_RUNFIRST):
                    a = _array(t.handle, mode, g, lvl, aid)
                    words += 0 if a is None else a.size
                if lvl >= 1 and ind is not None:
                    # entries of a level: per nonzero (COO, CSL, CSF leaf) or per fiber segment (CSF fiber levels);
                    # the CSF group's level arrays end with one sentinel entry
                    n = st["group_nnz"][g] if (g < 2 or lvl == order - 1) else st["segments"][lvl - 1]
                    gathered += np.unique(ind[:n]).size
            slices = st["group_slices"][g]
            assert got[name] == 4 * words + row * gathered + row * slices, (mode, name)
            want_total += 4 * words + row * gathered
        assert got["define"] == 4 * ((dims[mode] + 31) // 32) + row * (dims[mode] - owned_rows)
        assert got["total"] == want_total
        # what the roofline's numerator is made of: the B-CSF kernel's share is part of the total
        assert 0 < got["csf"] <= got["total"]
    t.close()
