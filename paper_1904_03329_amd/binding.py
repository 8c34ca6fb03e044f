"""ctypes binding of libhbcsf.so: the same entry points as include/hbcsf.h, argument marshalling only.

Every step of the MTTKRP path runs inside the library (host format builder and gfx950
kernels).  PyTorch is used by callers for device memory and streams only.  There is no
fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhbcsf.so")

HBCSF_MAX_ORDER = 5
ARR_IND, ARR_PTR, ARR_VAL, ARR_RUNFIRST, ARR_OWNED_BITS, ARR_COO_BITS, ARR_COO_PTR = 0, 1, 2, 3, 4, 5, 6
TUNE_SLICE_THRESHOLD, TUNE_PROFILE, TUNE_WAVES_PER_CU, TUNE_STEPS, TUNE_KERNEL_MASK = 0, 1, 2, 3, 4
TUNE_TRACE_BUFFER, TUNE_TRACE_CAPACITY, TUNE_PERSISTENT, TUNE_STREAM_BYTES, TUNE_FUSE_COO = 5, 6, 7, 8, 9
TUNE_DENSE_MID = 10
GROUP_COO, GROUP_CSL, GROUP_CSF = 0, 1, 2
OWNED_BIT = 0x80000000
ALS_KEEP_GRAMS = 1
ALS_LAZY_NORMALISATION = 2

EXPORTS = (
    "hbcsf_build_format", "hbcsf_device_bytes", "hbcsf_upload", "hbcsf_mttkrp", "hbcsf_mttkrp_f64", "hbcsf_get_stats",
    "hbcsf_host_array", "hbcsf_tune", "hbcsf_kernel_ms", "hbcsf_probe_row_gather", "hbcsf_free",
    "hbcsf_strerror", "hbcsf_last_error",
    "hbcsf_als_workspace_bytes", "hbcsf_als_create", "hbcsf_als_iteration", "hbcsf_als_normalise", "hbcsf_als_run", "hbcsf_als_phase_ms", "hbcsf_als_free", "hbcsf_sym_pinv",
    "hbcsf_gram_workspace_bytes", "hbcsf_gram", "hbcsf_gram_noalloc",
    "hbcsf_device_build_bytes", "hbcsf_build_format_device", "hbcsf_download", "hbcsf_relocate",
)


class hbcsf_opts(ctypes.Structure):
    _fields_ = [("fiber_threshold", ctypes.c_uint32), ("slice_threshold", ctypes.c_uint32),
                ("mode_order_policy", ctypes.c_uint32), ("group_mask", ctypes.c_uint32),
                ("hybrid_granularity", ctypes.c_uint32), ("coo_row_flags", ctypes.c_uint32),
                ("mid_blocking", ctypes.c_uint32), ("single_representation", ctypes.c_uint32)]


class hbcsf_stats(ctypes.Structure):
    _fields_ = [
        ("nnz", ctypes.c_uint64), ("slices", ctypes.c_uint64), ("fibers", ctypes.c_uint64 * (HBCSF_MAX_ORDER - 2)),
        ("segments", ctypes.c_uint64 * (HBCSF_MAX_ORDER - 2)), ("group_nnz", ctypes.c_uint64 * 3),
        ("group_slices", ctypes.c_uint64 * 3), ("shared_slices", ctypes.c_uint64),
        ("runs", ctypes.c_uint64 * 3), ("words_coo", ctypes.c_uint64), ("words_csf", ctypes.c_uint64),
        ("words_hbcsf", ctypes.c_uint64), ("stream_bytes", ctypes.c_uint64 * 3),
        ("distinct_rows", (ctypes.c_uint64 * HBCSF_MAX_ORDER) * 3), ("owned_rows", ctypes.c_uint64),
        ("flops_real", ctypes.c_uint64), ("level_mode", ctypes.c_uint32 * HBCSF_MAX_ORDER),
        ("fiber_threshold", ctypes.c_uint32), ("build_seconds", ctypes.c_double),
    ]


class HbcsfError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"hbcsf error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """Loads libhbcsf.so (built by paper_1904_03329_amd.build.build()); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run paper_1904_03329_amd.build.build() first")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int
        L.hbcsf_build_format.restype = i32
        L.hbcsf_build_format.argtypes = [i32, vp, u64, vp, vp, vp, ctypes.POINTER(vp)]
        L.hbcsf_device_bytes.restype = i32
        L.hbcsf_device_bytes.argtypes = [vp, ctypes.POINTER(u64)]
        L.hbcsf_upload.restype = i32
        L.hbcsf_upload.argtypes = [vp, vp, u64, vp]
        L.hbcsf_mttkrp.restype = i32
        L.hbcsf_mttkrp.argtypes = [vp, i32, i32, vp, vp, vp]
        L.hbcsf_mttkrp_f64.restype = i32
        L.hbcsf_mttkrp_f64.argtypes = [vp, i32, i32, vp, vp, vp]
        L.hbcsf_get_stats.restype = i32
        L.hbcsf_get_stats.argtypes = [vp, i32, ctypes.POINTER(hbcsf_stats)]
        L.hbcsf_host_array.restype = i32
        L.hbcsf_host_array.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(u64)]
        L.hbcsf_tune.restype = i32
        L.hbcsf_tune.argtypes = [vp, i32, u64]
        L.hbcsf_kernel_ms.restype = i32
        L.hbcsf_kernel_ms.argtypes = [vp, ctypes.c_uint32, ctypes.POINTER(ctypes.c_float * 4)]
        L.hbcsf_probe_row_gather.restype = i32
        L.hbcsf_probe_row_gather.argtypes = [vp, u64, vp, u64, i32, vp, vp, ctypes.POINTER(u64), ctypes.POINTER(u64)]
        L.hbcsf_free.restype = None
        L.hbcsf_free.argtypes = [vp]
        L.hbcsf_strerror.restype = ctypes.c_char_p
        L.hbcsf_strerror.argtypes = [i32]
        L.hbcsf_last_error.restype = ctypes.c_char_p
        L.hbcsf_last_error.argtypes = []
        L.hbcsf_als_workspace_bytes.restype = i32
        L.hbcsf_als_workspace_bytes.argtypes = [vp, i32, ctypes.POINTER(u64)]
        L.hbcsf_als_create.restype = i32
        L.hbcsf_als_create.argtypes = [vp, i32, vp, u64, ctypes.POINTER(vp)]
        L.hbcsf_als_iteration.restype = i32
        L.hbcsf_als_iteration.argtypes = [vp, vp, vp, i32, ctypes.POINTER(ctypes.c_double), vp]
        L.hbcsf_als_normalise.restype = i32
        L.hbcsf_als_normalise.argtypes = [vp, vp, vp]
        L.hbcsf_als_run.restype = i32
        L.hbcsf_als_run.argtypes = [vp, vp, vp, i32, ctypes.c_double, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double), vp]
        L.hbcsf_als_phase_ms.restype = i32
        L.hbcsf_als_phase_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float * 4)]
        L.hbcsf_device_build_bytes.restype = i32
        L.hbcsf_device_build_bytes.argtypes = [i32, vp, u64, vp, ctypes.POINTER(u64), ctypes.POINTER(u64)]
        L.hbcsf_build_format_device.restype = i32
        L.hbcsf_build_format_device.argtypes = [i32, vp, u64, vp, vp, vp, vp, u64, vp, u64, vp, ctypes.POINTER(vp)]
        L.hbcsf_relocate.restype = i32
        L.hbcsf_relocate.argtypes = [vp, vp, u64, vp]
        L.hbcsf_download.restype = i32
        L.hbcsf_download.argtypes = [vp, vp]
        L.hbcsf_gram_workspace_bytes.restype = i32
        L.hbcsf_gram_workspace_bytes.argtypes = [i32, ctypes.POINTER(u64)]
        L.hbcsf_gram.restype = i32
        L.hbcsf_gram.argtypes = [vp, u64, i32, vp, u64, vp, vp]
        L.hbcsf_gram_noalloc.restype = i32
        L.hbcsf_gram_noalloc.argtypes = [vp, u64, i32, vp, vp]
        L.hbcsf_sym_pinv.restype = i32
        L.hbcsf_sym_pinv.argtypes = [vp, i32, vp]
        L.hbcsf_als_free.restype = None
        L.hbcsf_als_free.argtypes = [vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise HbcsfError(rc, (lib().hbcsf_last_error() or b"").decode())


def build_format(dims, inds, vals, fiber_threshold=0, slice_threshold=0, mode_order_policy=0, group_mask=0,
                 hybrid_granularity=0, coo_row_flags=0, mid_blocking=0, single_representation=0):
    """hbcsf_build_format: host numpy index arrays (uint32) and values (float32) -> handle."""
    order = len(dims)
    d = np.asarray(dims, dtype=np.uint64)
    inds = [np.ascontiguousarray(x, dtype=np.uint32) for x in inds]
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    nnz = int(vals.shape[0])
    for x in inds:
        if x.shape[0] != nnz:
            raise ValueError("index arrays and vals must have the same length")
    ptrs = (ctypes.c_void_p * max(order, 1))(*[x.ctypes.data for x in inds])
    opts = hbcsf_opts(fiber_threshold, slice_threshold, mode_order_policy, group_mask, hybrid_granularity, coo_row_flags, mid_blocking, single_representation)
    h = ctypes.c_void_p()
    _check(lib().hbcsf_build_format(order, d.ctypes.data, nnz, ctypes.cast(ptrs, ctypes.c_void_p),
                                    vals.ctypes.data, ctypes.cast(ctypes.pointer(opts), ctypes.c_void_p),
                                    ctypes.byref(h)))
    return h


def _opts(fiber_threshold, slice_threshold, mode_order_policy, group_mask, hybrid_granularity=0, coo_row_flags=0, mid_blocking=0, single_representation=0):
    return hbcsf_opts(fiber_threshold, slice_threshold, mode_order_policy, group_mask, hybrid_granularity, coo_row_flags, mid_blocking, single_representation)


def device_build_bytes(dims, nnz: int, fiber_threshold=0, slice_threshold=0, mode_order_policy=0, group_mask=0,
                       hybrid_granularity=0, coo_row_flags=0, mid_blocking=0, single_representation=0):
    """hbcsf_device_build_bytes: (arena upper bound, workspace) in bytes."""
    d = np.asarray(dims, dtype=np.uint64)
    opts = _opts(fiber_threshold, slice_threshold, mode_order_policy, group_mask, hybrid_granularity, coo_row_flags, mid_blocking, single_representation)
    a, w = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().hbcsf_device_build_bytes(len(dims), d.ctypes.data, nnz,
                                          ctypes.cast(ctypes.pointer(opts), ctypes.c_void_p), ctypes.byref(a),
                                          ctypes.byref(w)))
    return int(a.value), int(w.value)


def build_format_device(dims, nnz: int, ind_ptrs, val_ptr: int, arena_ptr: int, arena_bytes: int, workspace_ptr: int,
                        workspace_bytes: int, stream: int = 0, fiber_threshold=0, slice_threshold=0,
                        mode_order_policy=0, group_mask=0, hybrid_granularity=0, coo_row_flags=0, mid_blocking=0, single_representation=0):
    """hbcsf_build_format_device: device addresses of the COO arrays in, resident handle out."""
    d = np.asarray(dims, dtype=np.uint64)
    opts = _opts(fiber_threshold, slice_threshold, mode_order_policy, group_mask, hybrid_granularity, coo_row_flags, mid_blocking, single_representation)
    ptrs = (ctypes.c_void_p * len(dims))(*[(p if p else None) for p in ind_ptrs])
    h = ctypes.c_void_p()
    _check(lib().hbcsf_build_format_device(len(dims), d.ctypes.data, nnz, ctypes.cast(ptrs, ctypes.c_void_p),
                                           ctypes.c_void_p(val_ptr or None),
                                           ctypes.cast(ctypes.pointer(opts), ctypes.c_void_p),
                                           ctypes.c_void_p(arena_ptr), arena_bytes, ctypes.c_void_p(workspace_ptr),
                                           workspace_bytes, ctypes.c_void_p(stream), ctypes.byref(h)))
    return h


def relocate(h, arena_ptr: int, nbytes: int, stream: int = 0):
    _check(lib().hbcsf_relocate(h, ctypes.c_void_p(arena_ptr), nbytes, ctypes.c_void_p(stream)))


def download(h, stream: int = 0):
    _check(lib().hbcsf_download(h, ctypes.c_void_p(stream)))


def device_bytes(h) -> int:
    n = ctypes.c_uint64()
    _check(lib().hbcsf_device_bytes(h, ctypes.byref(n)))
    return int(n.value)


def upload(h, arena_ptr: int, nbytes: int, stream: int = 0):
    """hbcsf_upload: arena_ptr is a device address (e.g. torch_tensor.data_ptr())."""
    _check(lib().hbcsf_upload(h, ctypes.c_void_p(arena_ptr), nbytes, ctypes.c_void_p(stream)))


def mttkrp(h, mode: int, rank: int, factor_ptrs, out_ptr: int, stream: int = 0):
    """hbcsf_mttkrp: factor_ptrs are device addresses (0 / None allowed at position `mode`)."""
    arr = (ctypes.c_void_p * len(factor_ptrs))(*[(p if p else None) for p in factor_ptrs])
    _check(lib().hbcsf_mttkrp(h, mode, rank, ctypes.cast(arr, ctypes.c_void_p), ctypes.c_void_p(out_ptr),
                              ctypes.c_void_p(stream)))


def mttkrp_f64(h, mode: int, rank: int, factor_ptrs, out_ptr: int, stream: int = 0):
    """hbcsf_mttkrp_f64: as mttkrp, the factor matrices and the output hold doubles."""
    arr = (ctypes.c_void_p * len(factor_ptrs))(*[(p if p else None) for p in factor_ptrs])
    _check(lib().hbcsf_mttkrp_f64(h, mode, rank, ctypes.cast(arr, ctypes.c_void_p), ctypes.c_void_p(out_ptr),
                                  ctypes.c_void_p(stream)))


def get_stats(h, mode: int) -> dict:
    st = hbcsf_stats()
    _check(lib().hbcsf_get_stats(h, mode, ctypes.byref(st)))
    out = {}
    for name, _ in hbcsf_stats._fields_:
        v = getattr(st, name)
        if name == "distinct_rows":
            v = [list(row) for row in v]
        elif hasattr(v, "__len__"):
            v = list(v)
        out[name] = v
    return out


def host_array(h, mode: int, group: int, level: int, array_id: int) -> np.ndarray:
    """Copy of one host-side format array (uint32, or float32 for ARR_VAL)."""
    p = ctypes.c_void_p()
    n = ctypes.c_uint64()
    _check(lib().hbcsf_host_array(h, mode, group, level, array_id, ctypes.byref(p), ctypes.byref(n)))
    ctype = ctypes.c_float if array_id == ARR_VAL else ctypes.c_uint32
    if n.value == 0:
        return np.zeros(0, dtype=np.float32 if array_id == ARR_VAL else np.uint32)
    buf = (ctype * n.value).from_address(p.value)
    return np.frombuffer(buf, dtype=np.float32 if array_id == ARR_VAL else np.uint32).copy()


def tune(h, key: int, value: int):
    _check(lib().hbcsf_tune(h, key, value))


def kernel_ms(h, calls_back: int = 0):
    """Milliseconds of the define / COO / CSL / CSF kernels of a profiled call."""
    ms = (ctypes.c_float * 4)()
    _check(lib().hbcsf_kernel_ms(h, calls_back, ctypes.byref(ms)))
    return [float(x) for x in ms]


def probe_row_gather(idx_ptr: int, n: int, table_ptr: int, table_rows: int, sink_ptr: int, stream: int = 0,
                     active_lane_groups: int = 8):
    """hbcsf_probe_row_gather: returns (rows the launch gathers, wavefront-level row-load instructions it issues)."""
    rows, instr = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().hbcsf_probe_row_gather(ctypes.c_void_p(idx_ptr), n, ctypes.c_void_p(table_ptr), table_rows,
                                        active_lane_groups, ctypes.c_void_p(sink_ptr), ctypes.c_void_p(stream),
                                        ctypes.byref(rows), ctypes.byref(instr)))
    return int(rows.value), int(instr.value)


def als_workspace_bytes(h, rank: int) -> int:
    n = ctypes.c_uint64()
    _check(lib().hbcsf_als_workspace_bytes(h, rank, ctypes.byref(n)))
    return int(n.value)


def als_create(h, rank: int, workspace_ptr: int, nbytes: int):
    """hbcsf_als_create: workspace_ptr is a device address."""
    a = ctypes.c_void_p()
    _check(lib().hbcsf_als_create(h, rank, ctypes.c_void_p(workspace_ptr), nbytes, ctypes.byref(a)))
    return a


def als_iteration(a, factor_ptrs, lambda_ptr: int = 0, flags: int = 0, want_fit: bool = True, stream: int = 0):
    """hbcsf_als_iteration: device addresses in, the fit (or None) out."""
    arr = (ctypes.c_void_p * len(factor_ptrs))(*factor_ptrs)
    fit = ctypes.c_double()
    _check(lib().hbcsf_als_iteration(a, ctypes.cast(arr, ctypes.c_void_p), ctypes.c_void_p(lambda_ptr or None), flags,
                                     ctypes.byref(fit) if want_fit else None, ctypes.c_void_p(stream)))
    return float(fit.value) if want_fit else None


def als_normalise(a, factor_ptrs, stream: int = 0):
    """hbcsf_als_normalise: carries out the put-off column normalisation on the factors (device addresses)."""
    arr = (ctypes.c_void_p * len(factor_ptrs))(*factor_ptrs)
    _check(lib().hbcsf_als_normalise(a, ctypes.cast(arr, ctypes.c_void_p), ctypes.c_void_p(stream or None)))


def als_run(a, factor_ptrs, lambda_ptr: int = 0, max_iterations: int = 50, tolerance: float = 1e-5, stream: int = 0):
    """hbcsf_als_run: returns (iterations done, fit)."""
    arr = (ctypes.c_void_p * len(factor_ptrs))(*factor_ptrs)
    done, fit = ctypes.c_int(), ctypes.c_double()
    _check(lib().hbcsf_als_run(a, ctypes.cast(arr, ctypes.c_void_p), ctypes.c_void_p(lambda_ptr or None), max_iterations,
                               tolerance, ctypes.byref(done), ctypes.byref(fit), ctypes.c_void_p(stream)))
    return int(done.value), float(fit.value)


def als_phase_ms(a):
    ms = (ctypes.c_float * 4)()
    _check(lib().hbcsf_als_phase_ms(a, ctypes.byref(ms)))
    return [float(x) for x in ms]


def gram_workspace_bytes(rank: int) -> int:
    n = ctypes.c_uint64(0)
    _check(lib().hbcsf_gram_workspace_bytes(rank, ctypes.byref(n)))
    return n.value


def gram(a_ptr: int, rows: int, rank: int, workspace_ptr: int, workspace_bytes: int, s_ptr: int, stream: int = 0):
    """hbcsf_gram: device addresses in; s_ptr receives the [rank][rank] fp64 Gram matrix."""
    _check(lib().hbcsf_gram(ctypes.c_void_p(a_ptr), rows, rank, ctypes.c_void_p(workspace_ptr), workspace_bytes,
                            ctypes.c_void_p(s_ptr), ctypes.c_void_p(stream or None)))


def gram_noalloc(a_ptr: int, rows: int, rank: int, s_ptr: int, stream: int = 0):
    """hbcsf_gram_noalloc: as gram, with the library's own scratch."""
    _check(lib().hbcsf_gram_noalloc(ctypes.c_void_p(a_ptr), rows, rank, ctypes.c_void_p(s_ptr),
                                    ctypes.c_void_p(stream or None)))


def sym_pinv(v: np.ndarray) -> np.ndarray:
    """hbcsf_sym_pinv: host fp64 symmetric matrix in, its pseudo-inverse out."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty_like(v)
    _check(lib().hbcsf_sym_pinv(v.ctypes.data, v.shape[0], out.ctypes.data))
    return out


def als_free(a):
    lib().hbcsf_als_free(a)


def free(h):
    lib().hbcsf_free(h)


def strerror(code: int) -> str:
    return lib().hbcsf_strerror(code).decode()


def last_error() -> str:
    return (lib().hbcsf_last_error() or b"").decode()
