"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

cfg2 is compared element by element.  cfg3-cfg5 are compared on sampled output rows that the oracle
computes one by one (the heaviest rows, random non-empty rows and empty rows), plus the cross-mode
invariant sum(M^(n) * A_n) = const, which holds at any size.
"""
import time

import numpy as np
import pytest

import gpu_util as GU

pytestmark = pytest.mark.gpu


def _run_workload(oracle, synth, name, full):
    import torch
    from paper_1904_03329_amd import HbcsfTensor

    t0 = time.time()
    t, facs, rank = synth.workload(name)
    print(f"{name}: generated nnz={t.nnz} draws={t.draws} in {time.time() - t0:.1f}s", flush=True)
    t0 = time.time()
    ht = HbcsfTensor(t.dims, t.inds, t.vals).to_device()
    print(f"{name}: built + uploaded in {time.time() - t0:.1f}s", flush=True)
    dfacs = [torch.from_numpy(f).cuda() for f in facs]
    rng = np.random.default_rng(99)
    invariant, scale = [], []
    for mode in range(t.order):
        out = torch.full((t.dims[mode], rank), float("nan"), dtype=torch.float32, device="cuda")
        ht.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), f"{name} mode {mode}: non-finite output"
        invariant.append(float((out.double() * dfacs[mode].double()).sum()))
        scale.append(float((out.double().abs() * dfacs[mode].double()).sum()))
        t0 = time.time()
        if full:
            want = oracle.mttkrp(t.dims, t.inds, t.vals, facs, mode)
            rel = GU.assert_close(out.cpu().numpy(), want, f"{name} mode {mode}")
        else:
            cnt = np.bincount(t.inds[mode], minlength=t.dims[mode])
            heavy = np.argsort(cnt)[-64:]
            nonempty = np.flatnonzero(cnt > 0)
            empty = np.flatnonzero(cnt == 0)
            rows = np.unique(np.concatenate([heavy, rng.choice(nonempty, size=min(4000, nonempty.size), replace=False),
                                             rng.choice(empty, size=min(500, empty.size), replace=False) if empty.size else heavy[:0]]))
            want = oracle.mttkrp_rows(t.dims, t.inds, t.vals, facs, mode, rows)
            got = out[torch.from_numpy(rows).cuda()].cpu().numpy()
            # the tolerance is relative to the largest entry of the whole result; the heaviest rows are in the sample
            rel = GU.assert_close(got, want, f"{name} mode {mode} ({rows.size} sampled rows)")
            if empty.size:
                assert float(out[torch.from_numpy(empty[:100000]).cuda()].abs().max()) == 0.0
        print(f"{name} mode {mode}: max|diff|/max|M| = {rel:.2e} (oracle {time.time() - t0:.1f}s)", flush=True)
        del out
    spread = (max(invariant) - min(invariant)) / max(scale)
    assert spread < 1e-5, f"{name}: cross-mode invariant differs by {spread:.2e}: {invariant}"
    ht.close()


def test_cfg2_every_element(oracle, synth):
    _run_workload(oracle, synth, "cfg2", full=True)


def test_cfg3_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg3", full=False)


def test_cfg4_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg4", full=False)


def test_cfg5_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg5", full=False)
