"""Seeded synthetic inputs (tensors, values, factor matrices) for tests and benchmarks.

This package only makes inputs.  It holds none of the MTTKRP arithmetic; the CPU
oracle and the GPU library are both fed from here and share nothing else.

The five workloads are stand-ins for the FROSTT / HaTen2 tensors of the paper's
Table III, which cannot be downloaded here: same orders (3 and 4), same scale
(up to 150 M nonzeros, dimensions up to tens of millions) and the strong
power-law skew of slice and fiber lengths that the paper's Table II quantifies.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsynthgen.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the generator (host C++ with OpenMP) into libsynthgen.so."""
    src = os.path.join(_HERE, "synthgen.cpp")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(
            ["g++", "-O3", "-march=x86-64-v2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", "-o", _SO, src]
        )
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(force=False)
        lib = ctypes.CDLL(_SO)
        lib.synth_tensor.restype = ctypes.c_int
        lib.synth_tensor.argtypes = [
            ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ]
        lib.synth_fill_uniform.restype = None
        lib.synth_fill_uniform.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                           ctypes.c_float, ctypes.c_float]
        lib.synth_scramble.restype = ctypes.c_uint64
        lib.synth_scramble.argtypes = [ctypes.c_uint64]
        lib.synth_unscramble.restype = ctypes.c_uint64
        lib.synth_unscramble.argtypes = [ctypes.c_uint64]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Workload:
    name: str
    dims: tuple
    nnz: int            # nominal number of stored nonzeros
    alpha: tuple        # Zipf exponent per mode; 0 = uniform
    rank: int
    seed: int
    topup: bool = True  # draw until `nnz` distinct coordinates exist

    @property
    def order(self) -> int:
        return len(self.dims)


# One entry per benchmark configuration, in the order the configurations are listed.
WORKLOADS = {
    "cfg1": Workload("cfg1", (100, 80, 60), 10_000, (0.0, 0.0, 0.0), 8, 1001),
    "cfg2": Workload("cfg2", (100_000, 100_000, 10_000), 5_000_000, (1.2, 1.2, 1.2), 32, 1002),
    "cfg3": Workload("cfg3", (480_000, 18_000, 2_000), 100_000_000, (1.5, 1.1, 1.1), 32, 1003),
    "cfg4": Workload("cfg4", (1_000_000, 50_000, 5_000, 1_000), 50_000_000, (1.3, 1.1, 1.0, 0.8), 32, 1004),
    "cfg5": Workload("cfg5", (40_000_000, 40_000_000, 1_000), 150_000_000, (1.05, 1.05, 0.0), 32, 1005),
}


@dataclass
class Tensor:
    dims: tuple
    inds: list           # order arrays of uint32 [nnz], 0-based
    vals: np.ndarray     # float32 [nnz]
    draws: int           # coordinates drawn before merging duplicates

    @property
    def nnz(self) -> int:
        return int(self.vals.shape[0])

    @property
    def order(self) -> int:
        return len(self.dims)


def tensor(dims, nnz, alpha, seed, topup=True) -> Tensor:
    """Distinct coordinates with per-mode bounded-Zipf (alpha>0) or uniform (alpha<=0) index
    laws over a seeded random permutation of each index range; values U[-1,1)."""
    lib = _load()
    order = len(dims)
    d = np.asarray(dims, dtype=np.uint64)
    a = np.asarray(alpha, dtype=np.float64)
    assert a.shape[0] == order
    inds = [np.empty(nnz, dtype=np.uint32) for _ in range(order)]
    vals = np.empty(nnz, dtype=np.float32)
    ptrs = (ctypes.c_void_p * order)(*[x.ctypes.data for x in inds])
    out_nnz = ctypes.c_uint64(0)
    out_draws = ctypes.c_uint64(0)
    rc = lib.synth_tensor(order, d.ctypes.data, a.ctypes.data, nnz, seed, 1 if topup else 0,
                          ctypes.cast(ptrs, ctypes.c_void_p), vals.ctypes.data,
                          ctypes.byref(out_nnz), ctypes.byref(out_draws))
    if rc != 0:
        raise RuntimeError(f"synth_tensor failed with code {rc}")
    n = out_nnz.value
    if n != nnz:
        inds = [x[:n].copy() for x in inds]
        vals = vals[:n].copy()
    return Tensor(tuple(int(x) for x in dims), inds, vals, int(out_draws.value))


def uniform(shape, seed, lo=0.0, hi=1.0) -> np.ndarray:
    """float32 array of U[lo,hi) values, a pure function of (seed, flat position)."""
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_uniform(out.ctypes.data, out.size, seed, lo, hi)
    return out


def factors(dims, rank, seed) -> list:
    """One row-major [dims[m], rank] float32 U[0,1) factor matrix per mode."""
    return [uniform((int(dims[m]), int(rank)), seed * 7919 + 31 * m + 17) for m in range(len(dims))]


def workload(name: str, scale: float = 1.0):
    """Tensor and factor matrices of a named workload.  `scale` < 1 shrinks every dimension
    and the nonzero count by that factor (same index laws) for quick experiments."""
    w = WORKLOADS[name]
    dims = tuple(max(2, int(round(x * scale))) for x in w.dims)
    nnz = max(1, int(round(w.nnz * scale)))
    t = tensor(dims, nnz, w.alpha, w.seed, w.topup)
    return t, factors(dims, w.rank, w.seed), w.rank


def structure(t: Tensor, mode: int) -> dict:
    """Slice-length statistics of one mode (printed beside benchmark results)."""
    cnt = np.bincount(t.inds[mode], minlength=t.dims[mode])
    nz = np.sort(cnt[cnt > 0])[::-1]
    top = max(1, int(round(0.001 * nz.size)))
    return {
        "slices": int(nz.size),
        "max_slice": int(nz[0]),
        "top0.1%_share": float(nz[:top].sum() / t.nnz),
        "singleton_slices": float((nz == 1).mean()),
        "slices_le2": float((nz <= 2).mean()),
        "slices_gt1e5": int((nz > 100_000).sum()),
        "stdev_nnz_per_slice": float(nz.std()),
    }
