"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

cfg2 is compared element by element.  cfg3-cfg5 are compared on sampled output rows that the oracle
computes one by one (the heaviest rows, random non-empty rows and empty rows), plus the cross-mode
invariant sum(M^(n) * A_n) = const, which holds at any size.  Each workload's format is then built again by
the device-side builder and compared, array for array, with the host-built one.
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
    del dfacs
    _device_build_matches(t, ht, name)
    ht.close()


def _device_build_matches(t, host, name):
    """The device-side builder must produce the host builder's arrays, which the checks above validated."""
    import torch
    from paper_1904_03329_amd import HbcsfTensor, binding as B

    t0 = time.time()
    di = [torch.from_numpy(x.view(np.int32)).cuda() for x in t.inds]
    dv = torch.from_numpy(t.vals).cuda()
    torch.cuda.synchronize()
    t1 = time.time()
    dev = HbcsfTensor.from_device_coo(t.dims, di, dv)
    torch.cuda.synchronize()
    print(f"{name}: device build {time.time() - t1:.2f}s (COO upload {t1 - t0:.2f}s)", flush=True)
    del di, dv
    assert B.device_bytes(dev.handle) == B.device_bytes(host.handle)
    B.download(dev.handle)
    for mode in range(t.order):
        sh, sd = host.stats(mode), dev.stats(mode)
        sh.pop("build_seconds"), sd.pop("build_seconds")
        assert sh == sd, f"{name} mode {mode}: statistics differ"
        for aid in (B.ARR_OWNED_BITS, B.ARR_COO_BITS, B.ARR_COO_PTR):
            assert np.array_equal(B.host_array(host.handle, mode, 0, 0, aid), B.host_array(dev.handle, mode, 0, 0, aid))
        for g in range(3):
            assert np.array_equal(B.host_array(host.handle, mode, g, 0, B.ARR_VAL).view(np.uint32),
                                  B.host_array(dev.handle, mode, g, 0, B.ARR_VAL).view(np.uint32)), (name, mode, g)
            for lvl in range(t.order):
                for aid in (B.ARR_IND, B.ARR_PTR, B.ARR_RUNFIRST):
                    try:
                        a = B.host_array(host.handle, mode, g, lvl, aid)
                    except B.HbcsfError:
                        continue
                    assert np.array_equal(a, B.host_array(dev.handle, mode, g, lvl, aid)), (name, mode, g, lvl, aid)
    dev.close()


def test_cfg2_every_element(oracle, synth):
    _run_workload(oracle, synth, "cfg2", full=True)


def test_cfg3_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg3", full=False)


def test_cfg4_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg4", full=False)


def test_cfg5_sampled_rows(oracle, synth):
    _run_workload(oracle, synth, "cfg5", full=False)
