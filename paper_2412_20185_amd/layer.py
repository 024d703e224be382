"""Offline preparation of one linear layer for the hot path, on the GPU.

Holds what DecDEC keeps per linear layer (Section 3.1, 4.1): the quantised
weights with their metadata in GPU memory and the residual R = W - W_hat in
pinned CPU memory.  The quantiser is the library's device kernel
(decdec_quantize_uniform); nothing here computes on the CPU.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class UniformLinear:
    """A K x N linear layer quantised to `bits` (3 or 4) with group-128 scales
    and zero points, plus its residual in pinned host memory: fp16 (rbits = 16)
    or the symmetric integer format of Section 4.2 with rbits = 4 (the paper's
    default), 2 or 8 bits per value and one fp16 scale per output column."""

    def __init__(self, W: np.ndarray | torch.Tensor, bits: int, keep_residual: bool = True, rbits: int = 16):
        if isinstance(W, np.ndarray):
            W = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32))
        Wd = W.to(device="cuda", dtype=torch.float32).contiguous()
        K, N = Wd.shape
        self.K, self.N, self.bits = K, N, bits
        self.rbits = rbits
        self.desc = B.Desc(K, N, bits, B.W_UNIFORM_G128, B.R_FMT_OF_BITS[rbits])
        nbytes = B.decdec_packed_bytes(self.desc)
        if nbytes == 0:
            raise ValueError("unsupported shape: K must be a multiple of 128 and N of 64")
        self.Wq = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.scales = torch.empty((K // 128, N), dtype=torch.float16, device="cuda")
        self.zeros = torch.empty((K // 128, N), dtype=torch.float16, device="cuda")
        want16 = keep_residual and rbits == 16
        R_dev = torch.empty((K, N), dtype=torch.float16, device="cuda") if want16 else None
        B.decdec_quantize_uniform(self.desc, Wd, self.Wq, self.scales, self.zeros, R_dev)
        torch.cuda.synchronize()
        self.R = self.R_scales = None
        if want16:
            self.R = torch.empty((K, N), dtype=torch.float16, pin_memory=True)
            self.R.copy_(R_dev)
        elif keep_residual:
            R32 = torch.empty((K, N), dtype=torch.float32, device="cuda")
            B.decdec_residual_f32(self.desc, Wd, self.Wq, self.scales, self.zeros, R32)
            self.R = torch.empty((K, N * rbits // 8), dtype=torch.uint8, pin_memory=True)
            self.R_scales = torch.empty(N, dtype=torch.float16, device="cuda")
            B.decdec_quantize_residual(K, N, rbits, R32, self.R, self.R_scales)
            torch.cuda.synchronize()
            del R32
        torch.cuda.synchronize()
        del Wd, R_dev

    def residual_to_device(self):
        """Moves the residual from pinned host memory into GPU memory (for a GPU with room for it:
        the same kernels then read the selected rows from HBM instead of over the host link)."""
        if self.R is not None and not self.R.is_cuda:
            self.R = self.R.cuda()
            torch.cuda.synchronize()
        return self

    def weight_bytes(self) -> int:
        """Algorithmic bytes the base GEMV has to move: packed codes, fp16 scales
        and zero points, x and y."""
        return self.K * self.N * self.bits // 8 + 4 * self.N * (self.K // 128) + 2 * self.K + 2 * self.N

    def residual_bytes(self, k: int) -> int:
        """Bytes that cross the host link for k selected channels (the column scales of the integer
        formats are kept in GPU memory, 2 N bytes, and do not cross it)."""
        return k * self.N * self.rbits // 8

    def gemv(self, x: torch.Tensor, k: int, y: torch.Tensor, ws: B.Workspace, stream=None):
        B.decdec_gemv(self.desc, x, self.Wq, self.scales, self.zeros, self.R, self.R_scales, k, y, ws, stream)


class LinearGroup:
    """Linear layers that consume the same activation vector (q/k/v, gate/up:
    the fused layer types of Section 4.4): one selection, one launch per kernel
    for the whole group through decdec_gemv_multi."""

    def __init__(self, linears, ys):
        self.linears = list(linears)
        self.ys = list(ys)
        self._arr = B.make_linears(
            (l.desc, l.Wq, l.scales, l.zeros, l.R, l.R_scales, y) for l, y in zip(self.linears, self.ys))

    def gemv(self, x: torch.Tensor, k: int, ws: B.Workspace, stream=None):
        B.decdec_gemv_multi(self._arr, x, k, ws, stream)
