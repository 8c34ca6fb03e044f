"""hbcsf_gram_noalloc (scratch held by the library, nothing allocated) against hbcsf_gram (caller's workspace)
and the fp64 oracle, through the C ABI: two calls in a row, the second on a smaller input, so that what the
first call left in the shared scratch would show.  Bar as for hbcsf_gram: 1e-5 * max |S|."""
import numpy as np
import pytest

from oracle import cpd_als
from paper_1904_03329_amd import binding as B

pytestmark = pytest.mark.gpu

TOL = 1e-5


def _both(a, rank):
    import torch

    rows = a.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    da = torch.from_numpy(a).cuda()
    n = B.gram_workspace_bytes(rank)
    ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    ref = torch.full((rank, rank), float("nan"), dtype=torch.float64, device="cuda")
    got = torch.full((rank, rank), float("nan"), dtype=torch.float64, device="cuda")
    B.gram(da.data_ptr(), rows, rank, ws.data_ptr(), n, ref.data_ptr(), stream)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.gram_noalloc(da.data_ptr(), rows, rank, got.data_ptr(), stream)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return got.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("rank", [32, 64, 8, 128, 16])
def test_two_calls_in_a_row_second_smaller(rank):
    rng = np.random.default_rng(900 + rank)
    big = rng.uniform(-1, 1, size=(700_001, rank)).astype(np.float32)
    small = rng.uniform(0, 1, size=(4_097, rank)).astype(np.float32)
    for a in (big, small, small[:1], big[:33]):
        print("gram_noalloc", a.shape, flush=True)
        got, ref = _both(a, rank)
        want = cpd_als.gram(a)
        scale = np.max(np.abs(want))
        assert np.all(np.isfinite(got))
        assert np.max(np.abs(got - ref)) <= TOL * scale, "differs from hbcsf_gram"
        assert np.max(np.abs(got - want)) <= TOL * scale, "differs from the oracle"
    if rank == 32:      # both entry points then run the same grid: equal bits
        got, ref = _both(big, rank)
        assert np.array_equal(got, ref)


def test_errors_and_empty_input():
    import torch

    a = torch.zeros((64, 32), device="cuda")
    s = torch.full((32, 32), float("nan"), dtype=torch.float64, device="cuda")
    for args in ((a.data_ptr(), 64, 24, s.data_ptr()), (0, 64, 32, s.data_ptr()), (a.data_ptr(), 64, 32, 0),
                 (a.data_ptr() + 4, 63, 32, s.data_ptr())):
        with pytest.raises(B.HbcsfError) as e:
            B.gram_noalloc(*args)
        assert e.value.code == -1
    B.gram_noalloc(a.data_ptr(), 0, 32, s.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(s.cpu().numpy(), np.zeros((32, 32)))
