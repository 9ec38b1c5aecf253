"""Thin binding of the offline entry point: allocates the outputs, marshals the arguments (no arithmetic here)."""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding


@dataclass
class QuantizedLayer:
    M: int
    N: int
    bits: int
    qidx: torch.Tensor      # uint8  [M * N * bits / 8]
    lut: torch.Tensor       # uint16 bit patterns as int16 [M, 2^bits]
    rowptr: torch.Tensor    # int32  [M + 1]
    cols: torch.Tensor      # int32  [capacity]; rowptr[M] entries are valid
    vals: torch.Tensor      # int16  [capacity] fp16 bit patterns
    iters: torch.Tensor     # int32  [M]

    def nnz(self) -> int:
        """Number of extracted entries (reads one integer back from the device)."""
        return int(self.rowptr[-1].item())


def quantize_layer(w: torch.Tensor, sens: torch.Tensor, bits: int, n_lo: int, n_hi: int, n_sens: int, max_iter: int = 32,
                   stream=None) -> QuantizedLayer:
    """w: fp16 bit patterns (int16 or float16 tensor) [M, N] on the GPU; sens: 16-bit sensitivities (int16 storage) [M, N]."""
    if not (w.is_cuda and sens.is_cuda):
        raise binding.SqllmError(8, "quantize_layer needs device tensors")
    M, N = w.shape
    dev = w.device
    cap = max(1, n_lo + n_hi + n_sens)
    ws_bytes = binding.sqllm_quantize_workspace_bytes(M, N)
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = QuantizedLayer(M=M, N=N, bits=bits,
                         qidx=torch.empty(M * N * bits // 8, dtype=torch.uint8, device=dev),
                         lut=torch.empty((M, 1 << bits), dtype=torch.int16, device=dev),
                         rowptr=torch.empty(M + 1, dtype=torch.int32, device=dev),
                         cols=torch.empty(cap, dtype=torch.int32, device=dev),
                         vals=torch.empty(cap, dtype=torch.int16, device=dev),
                         iters=torch.empty(M, dtype=torch.int32, device=dev))
    binding.sqllm_quantize_layer(M, N, bits, max_iter, w, sens, n_lo, n_hi, n_sens, workspace, ws_bytes,
                                 out.qidx, out.lut, out.rowptr, out.cols, out.vals, out.iters, stream)
    return out
