"""The seeded input generator: determinism, distinct coordinates, index laws (no GPU needed)."""
import os
import subprocess
import sys

import numpy as np


def _keys(t):
    k = np.zeros(t.nnz, dtype=np.int64)
    for m in range(t.order):
        k = k * t.dims[m] + t.inds[m]
    return k


def test_distinct_in_range_and_exact_count(synth):
    t = synth.tensor((500, 300, 40), 20_000, (1.2, 1.1, 0.0), seed=3)
    assert t.nnz == 20_000 and t.draws >= t.nnz
    assert np.unique(_keys(t)).shape[0] == t.nnz
    for m in range(3):
        assert t.inds[m].dtype == np.uint32 and int(t.inds[m].max()) < t.dims[m]
    assert t.vals.dtype == np.float32 and np.all(np.abs(t.vals) <= 1.0)
    assert abs(float(t.vals.mean())) < 0.05


def test_without_topup_draws_exactly_nnz(synth):
    t = synth.tensor((500, 300, 40), 20_000, (1.2, 1.1, 0.0), seed=3, topup=False)
    assert t.draws == 20_000 and t.nnz < 20_000
    assert np.unique(_keys(t)).shape[0] == t.nnz
    # the top-up tensor starts from the same draws, so it contains these coordinates
    full = synth.tensor((500, 300, 40), 20_000, (1.2, 1.1, 0.0), seed=3)
    assert np.isin(_keys(t), _keys(full)).all()


def test_same_seed_same_tensor_any_thread_count(synth):
    a = synth.tensor((2000, 50, 7, 3), 30_000, (1.3, 1.0, 0.8, 0.0), seed=11)
    code = (
        "import sys; sys.path.insert(0, %r); import synthgen, numpy as np;"
        "t = synthgen.tensor((2000, 50, 7, 3), 30000, (1.3, 1.0, 0.8, 0.0), seed=11);"
        "np.save(sys.argv[1], np.stack(t.inds + [t.vals.view(np.uint32)]))"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    import tempfile
    with tempfile.TemporaryDirectory() as d:
        p = os.path.join(d, "t.npy")
        env = dict(os.environ, OMP_NUM_THREADS="3")
        subprocess.check_call([sys.executable, "-c", code, p], env=env)
        b = np.load(p)
    assert np.array_equal(np.stack(a.inds + [a.vals.view(np.uint32)]), b)
    c = synth.tensor((2000, 50, 7, 3), 30_000, (1.3, 1.0, 0.8, 0.0), seed=12)
    assert not np.array_equal(a.inds[0], c.inds[0])


def test_zipf_law_matches_its_closed_form(synth):
    """With one long mode and no merging pressure, rank frequencies follow t^-alpha / H."""
    dim, alpha, n = 1000, 1.2, 400_000
    t = synth.tensor((dim, 1_000_000), n, (alpha, 0.0), seed=5)
    cnt = np.sort(np.bincount(t.inds[0], minlength=dim))[::-1].astype(np.float64)
    w = np.arange(1, dim + 1, dtype=np.float64) ** -alpha
    w /= w.sum()
    for k in (1, 10, 100):
        assert abs(cnt[:k].sum() / n - w[:k].sum()) < 0.01
    # the heavy index is not index 0: ranks go through a random permutation
    t2 = synth.tensor((dim, 1_000_000), n, (alpha, 0.0), seed=6)
    assert int(np.argmax(np.bincount(t.inds[0]))) != int(np.argmax(np.bincount(t2.inds[0])))


def test_uniform_fill_and_factors(synth):
    a = synth.uniform((1000, 32), seed=9)
    assert a.dtype == np.float32 and a.min() >= 0.0 and a.max() <= 1.0
    assert abs(float(a.mean()) - 0.5) < 0.01
    assert np.array_equal(a, synth.uniform((1000, 32), seed=9))
    f = synth.factors((10, 20, 30), 8, seed=1)
    assert [x.shape for x in f] == [(10, 8), (20, 8), (30, 8)]
    assert not np.array_equal(f[0], f[1][:10])


def test_scramble_is_a_bijection(synth):
    lib = synth._load()
    for x in [0, 1, 2**63, 2**64 - 1, 0x123456789abcdef]:
        assert lib.synth_unscramble(lib.synth_scramble(x)) == x
