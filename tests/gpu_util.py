"""Helpers for the GPU parity tests: run the library on a synthetic tensor and compare with the oracle."""
import numpy as np

from paper_1904_03329_amd import HbcsfTensor, binding as B

# Bar stated for this path: max |GPU - oracle| <= 1e-4 * max |oracle|, per mode, fp32 arithmetic.
REL_TOL = 1e-4
# fp64 entry point: both sides sum the same products in fp64 in different orders; a sum of n <= 10^7 terms carries a
# rounding error of order sqrt(n) * 2^-53 ~ 4e-13 of the terms' magnitude on each side.
REL_TOL_F64 = 1e-12


def gpu_mttkrp_all_modes(dims, inds, vals, facs, tune_ts=None, tune_dense=None, tune_steps=None, tune_fuse=None,
                         **opts):
    """Returns (list of float32 numpy results per mode, per-mode stats)."""
    import torch

    t = HbcsfTensor(dims, inds, vals, **opts).to_device()
    if tune_ts is not None:
        B.tune(t.handle, B.TUNE_SLICE_THRESHOLD, tune_ts)
    if tune_dense is not None:
        B.tune(t.handle, B.TUNE_DENSE_MID, tune_dense)
    if tune_steps is not None:
        B.tune(t.handle, B.TUNE_STEPS, tune_steps)
    if tune_fuse is not None:
        B.tune(t.handle, B.TUNE_FUSE_COO, tune_fuse)
    dfacs = [torch.from_numpy(np.ascontiguousarray(f)).cuda() for f in facs]
    outs, stats = [], []
    for mode in range(len(dims)):
        rank = facs[(mode + 1) % len(dims)].shape[1]
        out = torch.full((dims[mode], rank), float("nan"), dtype=dfacs[0].dtype, device="cuda")
        t.mttkrp(mode, dfacs, out)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        stats.append(t.stats(mode))
    t.close()
    return outs, stats


def assert_close(got, want, what="", tol=REL_TOL):
    scale = float(np.max(np.abs(want))) if want.size else 0.0
    err = float(np.max(np.abs(got.astype(np.float64) - want))) if want.size else 0.0
    assert np.all(np.isfinite(got)), f"{what}: non-finite values in the GPU result"
    assert err <= tol * max(scale, 1e-30), f"{what}: max|diff| {err:.3e} > {tol} * max|M| {scale:.3e}"
    return err / max(scale, 1e-30)
