"""TEST INFRASTRUCTURE ONLY: Python access to the plain CPU oracle (mttkrp_oracle.c).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
The product (paper_1904_03329_amd) never does, and this package never imports the product.

The oracle is the plain definition of mode-n MTTKRP (Section II-C, Eq. 4-7; Algorithm
"COO-MTTKRP"): M[i_n][r] += v * prod_{m != n} A_m[i_m][r], accumulated in fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle_mttkrp.so")
_SO_OMP = os.path.join(_HERE, "liboracle_mttkrp_omp.so")
_lib = None
_lib_omp = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc: -O2, no fast-math, single thread; and, as a library of its own, the same
    loop on all cores (mttkrp_oracle_omp.c, -fopenmp), which only the benchmark's CPU baseline uses."""
    for so, name, extra in ((_SO, "mttkrp_oracle.c", []), (_SO_OMP, "mttkrp_oracle_omp.c", ["-fopenmp"])):
        src = os.path.join(_HERE, name)
        if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
            subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC"] + extra + ["-o", so, src])
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(force=False)
        lib = ctypes.CDLL(_SO)
        lib.oracle_mttkrp.restype = ctypes.c_int
        lib.oracle_mttkrp.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_void_p]
        lib.oracle_mttkrp_f64.restype = ctypes.c_int
        lib.oracle_mttkrp_f64.argtypes = lib.oracle_mttkrp.argtypes
        lib.oracle_mttkrp_rows.restype = ctypes.c_int
        lib.oracle_mttkrp_rows.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
        _lib = lib
    return _lib


def _marshal(dims, inds, vals, factors, mode, fdtype=np.float32):
    order = len(dims)
    if len(inds) != order or len(factors) != order:
        raise ValueError("need one index array and one factor matrix per mode")
    inds = [np.ascontiguousarray(x, dtype=np.uint32) for x in inds]
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    nnz = vals.shape[0]
    rank = None
    facs = []
    for m in range(order):
        if m == mode:
            facs.append(None)
            continue
        f = np.ascontiguousarray(factors[m], dtype=fdtype)
        if f.ndim != 2 or f.shape[0] != dims[m]:
            raise ValueError(f"factor {m} must be [{dims[m]}, R]")
        rank = f.shape[1] if rank is None else rank
        if f.shape[1] != rank:
            raise ValueError("factor matrices disagree on R")
        facs.append(f)
    d = np.asarray(dims, dtype=np.uint64)
    iptr = (ctypes.c_void_p * order)(*[x.ctypes.data for x in inds])
    fptr = (ctypes.c_void_p * order)(*[(f.ctypes.data if f is not None else None) for f in facs])
    keep = (inds, vals, facs, d)
    return order, d, nnz, iptr, vals, rank, fptr, keep


def mttkrp(dims, inds, vals, factors, mode) -> np.ndarray:
    """fp64 [dims[mode], R] mode-`mode` MTTKRP of the COO tensor (0-based mode)."""
    order, d, nnz, iptr, vals, rank, fptr, keep = _marshal(dims, inds, vals, factors, mode)
    out = np.empty((int(dims[mode]), rank), dtype=np.float64)
    rc = _load().oracle_mttkrp(order, d.ctypes.data, nnz, ctypes.cast(iptr, ctypes.c_void_p),
                               vals.ctypes.data, rank, ctypes.cast(fptr, ctypes.c_void_p), mode,
                               out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_mttkrp failed with code {rc}")
    return out


def mttkrp_f64(dims, inds, vals, factors, mode) -> np.ndarray:
    """The same sum with fp64 factor matrices (the values stay fp32): fp64 [dims[mode], R]."""
    order, d, nnz, iptr, vals, rank, fptr, keep = _marshal(dims, inds, vals, factors, mode, np.float64)
    out = np.empty((int(dims[mode]), rank), dtype=np.float64)
    rc = _load().oracle_mttkrp_f64(order, d.ctypes.data, nnz, ctypes.cast(iptr, ctypes.c_void_p),
                                   vals.ctypes.data, rank, ctypes.cast(fptr, ctypes.c_void_p), mode,
                                   out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_mttkrp_f64 failed with code {rc}")
    return out


def mttkrp_rows(dims, inds, vals, factors, mode, rows) -> np.ndarray:
    """fp64 [len(rows), R]: the rows `rows` (distinct) of the mode-`mode` MTTKRP."""
    order, d, nnz, iptr, vals, rank, fptr, keep = _marshal(dims, inds, vals, factors, mode)
    rows = np.asarray(rows, dtype=np.int64)
    slot = np.full(int(dims[mode]), -1, dtype=np.int32)
    slot[rows] = np.arange(rows.shape[0], dtype=np.int32)
    out = np.empty((rows.shape[0], rank), dtype=np.float64)
    rc = _load().oracle_mttkrp_rows(order, d.ctypes.data, nnz, ctypes.cast(iptr, ctypes.c_void_p),
                                    vals.ctypes.data, rank, ctypes.cast(fptr, ctypes.c_void_p), mode,
                                    slot.ctypes.data, rows.shape[0], out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_mttkrp_rows failed with code {rc}")
    return out


def mttkrp_all_cores(dims, inds, vals, factors, mode):
    """The oracle's loop split over all host cores with atomic fp64 adds (for the benchmark's reported CPU
    baseline; not the parity reference).  Returns (fp64 [dims[mode], R], threads used)."""
    global _lib_omp
    if _lib_omp is None:
        if not os.path.exists(_SO_OMP):
            build(force=False)
        lib = ctypes.CDLL(_SO_OMP)
        lib.oracle_mttkrp_omp.restype = ctypes.c_int
        lib.oracle_mttkrp_omp.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                          ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
        _lib_omp = lib
    order, d, nnz, iptr, vals, rank, fptr, keep = _marshal(dims, inds, vals, factors, mode)
    out = np.empty((int(dims[mode]), rank), dtype=np.float64)
    team = ctypes.c_int(0)
    rc = _lib_omp.oracle_mttkrp_omp(order, d.ctypes.data, nnz, ctypes.cast(iptr, ctypes.c_void_p),
                                    vals.ctypes.data, rank, ctypes.cast(fptr, ctypes.c_void_p), mode,
                                    out.ctypes.data, ctypes.byref(team))
    if rc != 0:
        raise RuntimeError(f"oracle_mttkrp_omp failed with code {rc}")
    return out, team.value
