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
    and zero points, plus its fp16 residual in pinned host memory."""

    def __init__(self, W: np.ndarray | torch.Tensor, bits: int, keep_residual: bool = True):
        if isinstance(W, np.ndarray):
            W = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32))
        Wd = W.to(device="cuda", dtype=torch.float32).contiguous()
        K, N = Wd.shape
        self.K, self.N, self.bits = K, N, bits
        self.desc = B.Desc(K, N, bits, B.W_UNIFORM_G128, B.R_FP16)
        nbytes = B.decdec_packed_bytes(self.desc)
        if nbytes == 0:
            raise ValueError("unsupported shape: K must be a multiple of 128 and N of 64")
        self.Wq = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.scales = torch.empty((K // 128, N), dtype=torch.float16, device="cuda")
        self.zeros = torch.empty((K // 128, N), dtype=torch.float16, device="cuda")
        R_dev = torch.empty((K, N), dtype=torch.float16, device="cuda") if keep_residual else None
        B.decdec_quantize_uniform(self.desc, Wd, self.Wq, self.scales, self.zeros, R_dev)
        torch.cuda.synchronize()
        self.R = None
        if keep_residual:
            self.R = torch.empty((K, N), dtype=torch.float16, pin_memory=True)
            self.R.copy_(R_dev)
            torch.cuda.synchronize()
        del Wd, R_dev

    def weight_bytes(self) -> int:
        """Algorithmic bytes the base GEMV has to move: packed codes, fp16 scales
        and zero points, x and y."""
        return self.K * self.N * self.bits // 8 + 4 * self.N * (self.K // 128) + 2 * self.K + 2 * self.N

    def residual_bytes(self, k: int) -> int:
        return k * self.N * 2

    def gemv(self, x: torch.Tensor, k: int, y: torch.Tensor, ws: B.Workspace, stream=None):
        B.decdec_gemv(self.desc, x, self.Wq, self.scales, self.zeros, self.R, None, k, y, ws, stream)


class LinearGroup:
    """Linear layers that consume the same activation vector (q/k/v, gate/up:
    the fused layer types of Section 4.4): one selection, one launch per kernel
    for the whole group through decdec_gemv_multi."""

    def __init__(self, linears, ys):
        self.linears = list(linears)
        self.ys = list(ys)
        self._arr = B.make_linears(
            (l.desc, l.Wq, l.scales, l.zeros, l.R, None, y) for l, y in zip(self.linears, self.ys))

    def gemv(self, x: torch.Tensor, k: int, ws: B.Workspace, stream=None):
        B.decdec_gemv_multi(self._arr, x, k, ws, stream)
