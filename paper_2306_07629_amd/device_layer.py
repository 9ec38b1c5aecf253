"""A quantised layer resident in HBM: torch tensors as owners of device memory, nothing more."""
from __future__ import annotations

import numpy as np

from . import binding as _b


class DeviceLayer:
    """Uploads the arrays of a generated layer (any object with M, N, bits, B, nnz, qidx, lut, rowptr, cols,
    vals, x as numpy arrays; fp16 data as uint16 bit patterns) and calls the library on them."""

    def __init__(self, layer, device="cuda:0"):
        import torch
        self.torch = torch
        self.M, self.N, self.bits, self.B, self.nnz = layer.M, layer.N, layer.bits, layer.B, int(layer.nnz)
        dev = torch.device(device)
        up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a).view(dt)).to(dev)
        self.qidx = up(layer.qidx, np.uint8)
        self.lut = up(layer.lut, np.int16)
        self.rowptr = up(layer.rowptr, np.int32)
        self.cols = up(layer.cols, np.int32) if self.nnz else None
        self.vals = up(layer.vals, np.int16) if self.nnz else None
        self.x = up(layer.x, np.int16)
        self.y = torch.zeros((self.M, self.B), dtype=torch.int16, device=dev)
        self.plan = None

    def build_plan(self, stream=None):
        """One-time re-layout of the CSR arrays for the one-column kernel (sqllm_csr_plan_build); matvec() then passes it on."""
        if self.nnz and self.plan is None:
            nbytes = _b.sqllm_csr_plan_bytes(self.M, self.N, self.nnz)
            self.plan = self.torch.empty(nbytes, dtype=self.torch.uint8, device=self.qidx.device)
            _b.sqllm_csr_plan_build(self.M, self.N, self.nnz, self.rowptr, self.cols, self.vals, self.plan, nbytes, stream)
        return self

    def clone_weights(self):
        """A second copy of the weight arrays at different addresses (for cold-cache timing)."""
        other = object.__new__(DeviceLayer)
        other.__dict__.update(self.__dict__)
        other.qidx = self.qidx.clone(); other.lut = self.lut.clone(); other.rowptr = self.rowptr.clone()
        other.cols = None if self.cols is None else self.cols.clone()
        other.vals = None if self.vals is None else self.vals.clone()
        other.plan = None if self.plan is None else self.plan.clone()
        other.y = self.y.clone()
        return other

    # --- library calls (each enqueues on the current stream)
    def matvec(self, stream=None):
        _b.sqllm_dense_sparse_matvec(self.M, self.N, self.bits, self.nnz, self.B, self.qidx, self.lut, self.rowptr,
                                     self.cols, self.vals, self.x, self.y, stream, plan=self.plan)
        return self.y

    def descriptor(self):
        """the tuple binding.layer_descriptors() takes (one activation column)"""
        return (self.M, self.N, self.bits, self.nnz, self.qidx, self.lut, self.rowptr, self.cols, self.vals, self.x, self.y, self.plan)

    def lut_gemv(self, accumulate=0, stream=None):
        _b.sqllm_lut_gemv(self.M, self.N, self.bits, self.B, self.qidx, self.lut, self.x, self.y, accumulate, stream)
        return self.y

    def csr_spmv(self, accumulate=0, rowwise=False, stream=None):
        f = _b.sqllm_csr_spmv_rowwise if rowwise else _b.sqllm_csr_spmv
        f(self.M, self.N, self.nnz, self.B, self.rowptr, self.cols, self.vals, self.x, self.y, accumulate, stream)
        return self.y

    def unpack(self):
        out = self.torch.empty((self.M, self.N), dtype=self.torch.uint8, device=self.qidx.device)
        _b.sqllm_unpack_indices(self.M, self.N, self.bits, self.qidx, out)
        return out

    def dequantize(self):
        out = self.torch.empty((self.M, self.N), dtype=self.torch.int16, device=self.qidx.device)
        _b.sqllm_dequantize(self.M, self.N, self.bits, self.qidx, self.lut, out)
        return out

    def y_host(self) -> np.ndarray:
        """y as float64 [M, B] (device fp16 bit patterns decoded on the host)."""
        self.torch.cuda.synchronize()
        return self.y.cpu().numpy().view(np.float16).astype(np.float64)
