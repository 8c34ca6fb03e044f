"""MI355X-native sparse MTTKRP with a load-balanced hybrid CSF format (HB-CSF).

`binding` mirrors the C ABI of include/hbcsf.h one to one.  `HbcsfTensor` is a small
convenience wrapper that lets PyTorch supply device memory and the current stream; all
computation happens in libhbcsf.so.
"""
from __future__ import annotations

from . import binding

__all__ = ["binding", "HbcsfTensor", "CpdAls"]


class HbcsfTensor:
    """A sparse tensor built into per-mode HB-CSF, optionally resident on the current GPU."""

    def __init__(self, dims, inds, vals, **opts):
        self.dims = tuple(int(d) for d in dims)
        self.order = len(self.dims)
        self.handle = binding.build_format(self.dims, inds, vals, **opts)
        self._arena = None

    @classmethod
    def from_device_coo(cls, dims, inds, vals, compact: bool = True, **opts):
        """Builds the format on the GPU from CUDA tensors (int32 / uint32-valued index tensors of dtype
        torch.int32, float32 values); the result is resident.  With `compact` the arrays are moved from the
        upper-bound arena the build needs into one of exactly their size."""
        import torch

        self = cls.__new__(cls)
        self.dims = tuple(int(d) for d in dims)
        self.order = len(self.dims)
        self.handle = None
        self._arena = None
        nnz = int(vals.shape[0])
        for x in list(inds) + [vals]:
            if not x.is_cuda or not x.is_contiguous() or x.shape[0] != nnz:
                raise ValueError("index and value tensors must be contiguous CUDA tensors of one length")
        if vals.dtype != torch.float32 or any(x.dtype != torch.int32 for x in inds):
            raise ValueError("indices must be torch.int32 and values torch.float32")
        stream = torch.cuda.current_stream().cuda_stream
        arena_bytes, ws_bytes = binding.device_build_bytes(self.dims, nnz, **opts)
        arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        self.handle = binding.build_format_device(self.dims, nnz, [x.data_ptr() for x in inds], vals.data_ptr(),
                                                  arena.data_ptr(), arena_bytes, ws.data_ptr(), ws_bytes, stream, **opts)
        del ws
        if compact:
            used = max(binding.device_bytes(self.handle), 256)
            small = torch.empty(used, dtype=torch.uint8, device="cuda")
            binding.relocate(self.handle, small.data_ptr(), used, stream)
            arena = small
        self._arena = arena
        return self

    def stats(self, mode: int) -> dict:
        return binding.get_stats(self.handle, mode)

    def to_device(self):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: hbcsf_upload needs a HIP device")
        n = binding.device_bytes(self.handle)
        self._arena = torch.empty(max(n, 256), dtype=torch.uint8, device="cuda")
        binding.upload(self.handle, self._arena.data_ptr(), self._arena.numel(),
                       torch.cuda.current_stream().cuda_stream)
        return self

    def mttkrp(self, mode: int, factors, out=None):
        """factors: one CUDA [dims[m], R] tensor per mode (entry `mode` may be None), all float32 or all float64
        (float64: fp64 partial sums and output, hbcsf_mttkrp_f64)."""
        import torch

        rank = None
        dtype = None
        ptrs = []
        for m in range(self.order):
            f = factors[m]
            if m == mode or f is None:
                ptrs.append(0)
                continue
            dtype = f.dtype if dtype is None else dtype
            if f.dtype not in (torch.float32, torch.float64) or f.dtype != dtype or not f.is_cuda or not f.is_contiguous():
                raise ValueError("factors must be contiguous CUDA tensors, all float32 or all float64")
            if f.shape[0] != self.dims[m]:
                raise ValueError(f"factor {m} must have {self.dims[m]} rows")
            rank = f.shape[1] if rank is None else rank
            if f.shape[1] != rank:
                raise ValueError("factor matrices disagree on the rank")
            ptrs.append(f.data_ptr())
        if out is None:
            out = torch.empty((self.dims[mode], rank), dtype=dtype, device="cuda")
        elif (out.dtype != dtype or not out.is_cuda or not out.is_contiguous()
              or tuple(out.shape) != (self.dims[mode], rank)):
            raise ValueError("out must be a contiguous CUDA tensor [dims[mode], R] of the factors' dtype")
        call = binding.mttkrp_f64 if dtype == torch.float64 else binding.mttkrp
        call(self.handle, mode, rank, ptrs, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        return out

    def close(self):
        if self.handle is not None:
            binding.free(self.handle)
            self.handle = None
        self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class CpdAls:
    """CPD-ALS iterations on a device-resident HbcsfTensor; PyTorch supplies the workspace and the stream."""

    def __init__(self, tensor: HbcsfTensor, rank: int):
        import torch

        self.tensor = tensor
        self.rank = int(rank)
        n = binding.als_workspace_bytes(tensor.handle, self.rank)
        self._ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        self.handle = binding.als_create(tensor.handle, self.rank, self._ws.data_ptr(), n)
        self.lam = torch.ones(self.rank, dtype=torch.float32, device="cuda")

    def iteration(self, factors, keep_grams: bool = False, lazy: bool = False) -> float:
        """Updates the CUDA float32 factor matrices in place, stores lambda in self.lam, returns the fit.
        lazy: the closing column normalisation may be put off (see normalise)."""
        import torch

        for m, f in enumerate(factors):
            if (f.dtype != torch.float32 or not f.is_cuda or not f.is_contiguous()
                    or tuple(f.shape) != (self.tensor.dims[m], self.rank)):
                raise ValueError(f"factor {m} must be a contiguous float32 CUDA tensor [{self.tensor.dims[m]}, {self.rank}]")
        return binding.als_iteration(self.handle, [f.data_ptr() for f in factors], self.lam.data_ptr(),
                                     (binding.ALS_KEEP_GRAMS if keep_grams else 0)
                                     | (binding.ALS_LAZY_NORMALISATION if lazy else 0), True,
                                     torch.cuda.current_stream().cuda_stream)

    def normalise(self, factors):
        """Writes the unit-norm factors after iterations with lazy=True."""
        import torch

        binding.als_normalise(self.handle, [f.data_ptr() for f in factors], torch.cuda.current_stream().cuda_stream)

    def run(self, factors, max_iterations: int = 50, tolerance: float = 1e-5):
        """Iterates until the fit changes by less than `tolerance`; returns (iterations done, fit)."""
        import torch

        return binding.als_run(self.handle, [f.data_ptr() for f in factors], self.lam.data_ptr(), max_iterations,
                               tolerance, torch.cuda.current_stream().cuda_stream)

    def phase_ms(self):
        return binding.als_phase_ms(self.handle)

    def close(self):
        if self.handle is not None:
            binding.als_free(self.handle)
            self.handle = None
        self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
