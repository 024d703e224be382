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


class StoredLinear:
    """A linear layer whose stored parameters are given, not produced here: packed weights with their
    metadata in GPU memory and residual rows in pinned host memory, in the library's formats.  Used for
    timing on shapes whose offline preparation is not the point (the kernels' speed does not depend on the
    values), with parameters drawn at random."""

    def __init__(self, desc, Wq, scales, zeros_or_lut, R, R_scales, rbits: int):
        self.desc, self.Wq, self.scales, self.zeros, self.R, self.R_scales = desc, Wq, scales, zeros_or_lut, R, R_scales
        self.K, self.N, self.bits, self.rbits = desc.K, desc.N, desc.wbits, rbits

    @staticmethod
    def random_residual(K: int, N: int, rbits: int, seed: int):
        """(pinned rows, device column scales or None) with random contents; fp16 payloads are kept finite."""
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        R = torch.empty((K, N * rbits // 8), dtype=torch.uint8, pin_memory=True)
        if rbits == 16:
            R.view(torch.float16).copy_((torch.randn((K, N), device="cuda", generator=g) * 0.003).half())
            return R, None
        R.copy_(torch.randint(0, 256, R.shape, dtype=torch.uint8, device="cuda", generator=g))
        return R, torch.full((N,), 1e-3, dtype=torch.float16, device="cuda")

    @classmethod
    def like(cls, lin, rbits: int, seed: int = 0):
        """The weights of `lin` (shared, not copied) with a random residual of another format."""
        desc = B.Desc(lin.K, lin.N, lin.bits, lin.desc.wfmt, B.R_FMT_OF_BITS[rbits])
        R, Rs = cls.random_residual(lin.K, lin.N, rbits, seed)
        return cls(desc, lin.Wq, lin.scales, lin.zeros, R, Rs, rbits)

    @classmethod
    def random(cls, K: int, N: int, wbits: int, wfmt: int, rbits: int, seed: int = 0):
        desc = B.Desc(K, N, wbits, wfmt, B.R_FMT_OF_BITS[rbits])
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        Wq = torch.randint(0, 256, (B.decdec_packed_bytes(desc),), dtype=torch.uint8, device="cuda", generator=g)
        if wfmt == B.W_UNIFORM_G128:
            sc = torch.full((K // 128, N), 0.01, dtype=torch.float16, device="cuda")
            zl = torch.full((K // 128, N), 3.0, dtype=torch.float16, device="cuda")
        else:
            sc = None
            zl = (torch.sort(torch.randn(N, 8, device="cuda", generator=g), dim=1).values * 0.02).half().contiguous()
        R, Rs = cls.random_residual(K, N, rbits, seed + 1)
        return cls(desc, Wq, sc, zl, R, Rs, rbits)

    def weight_bytes(self) -> int:
        meta = 4 * self.N * (self.K // 128) if self.desc.wfmt == B.W_UNIFORM_G128 else 16 * self.N
        return self.K * self.N * self.bits // 8 + meta + 2 * self.K + 2 * self.N

    def residual_bytes(self, k: int) -> int:
        return k * self.N * self.rbits // 8

    def gemv(self, x: torch.Tensor, k: int, y: torch.Tensor, ws: B.Workspace, stream=None):
        B.decdec_gemv(self.desc, x, self.Wq, self.scales, self.zeros, self.R, self.R_scales, k, y, ws, stream)


def random_layer(shapes, wbits: int, wfmt: int, rbits: int, order, ys, seed: int = 0):
    """One decoder layer of random stored parameters: for every (input, [names]) of `order` the array of
    decdec_linear for decdec_gemv_multi, writing to ys[name]."""
    lin = {name: StoredLinear.random(K, N, wbits, wfmt, rbits, seed=1000 * seed + 2 * j)
           for j, (name, K, N, _) in enumerate(shapes)}
    out = []
    for _, names in order:
        arr = B.make_linears([(lin[n].desc, lin[n].Wq, lin[n].scales, lin[n].zeros, lin[n].R, lin[n].R_scales, ys[n])
                              for n in names])
        out.append(arr)
    return out


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
