"""Shared test plumbing: turn oracle artefacts into device tensors, run the
HIP path through the C ABI binding, and compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2412_20185_amd as dd

RBITS = {"int2": 2, "int4": 4, "int8": 8}
RFMT = {"fp16": dd.R_FP16, "int4": dd.R_INT4_SYM_COL, "int2": dd.R_INT2_SYM_COL, "int8": dd.R_INT8_SYM_COL}
TOL_Y = 2e-3          # max relative error of y against the fp64 oracle (floor 1 % of rms on the denominator)


class Problem:
    """One linear layer prepared for both sides from the oracle's artefacts."""

    def __init__(self, W: np.ndarray, bits: int, wfmt: str = "uniform", rfmt: str = "fp16",
                 lut_iters: int = 16, alphas=None, keep_dense: bool = True):
        K, N = W.shape
        self.K, self.N, self.bits = K, N, bits
        self.W = W
        if wfmt == "uniform":
            self.codes, self.scales, self.zeros = oracle.quantize_uniform(W, bits)
            self.lut = None
            W_hat = oracle.dequantize_uniform(self.codes, self.scales, self.zeros)
            self.desc = dd.Desc(K, N, bits, dd.W_UNIFORM_G128, RFMT[rfmt])
        else:
            self.codes, self.lut = oracle.quantize_lut(W, iters=lut_iters)
            self.scales = self.zeros = None
            W_hat = oracle.dequantize_lut(self.codes, self.lut)
            self.desc = dd.Desc(K, N, 3, dd.W_LUT_COL8, RFMT[rfmt])
        if rfmt == "fp16":
            self.R = oracle.residual_fp16(W, W_hat)
            self.R_real = self.R
            self.Rq = self.Rs = None
        else:
            kw = {} if alphas is None else {"alphas": alphas}
            self.Rq, self.Rs = oracle.quantize_residual_sym(W.astype(np.float64) - W_hat, RBITS[rfmt], **kw)
            self.R_real = oracle.dequantize_residual_int4(self.Rq, self.Rs)
            self.R = None
        self.W_hat = W_hat if keep_dense else None
        self.rfmt = rfmt
        self._dev = None

    def device(self):
        if self._dev is None:
            packed = dd.decdec_pack_weights(self.desc, self.codes)
            d = {"Wq": torch.from_numpy(packed).cuda()}
            if self.lut is None:
                d["scales"] = torch.from_numpy(self.scales).cuda()
                d["zl"] = torch.from_numpy(self.zeros).cuda()
            else:
                d["scales"] = None
                d["zl"] = torch.from_numpy(self.lut).cuda()
            if self.rfmt == "fp16":
                d["R"] = torch.from_numpy(self.R).pin_memory()
                d["Rs"] = None
            else:
                d["R"] = torch.from_numpy(dd.decdec_pack_residual_int(self.Rq, RBITS[self.rfmt])).pin_memory()
                d["Rs"] = torch.from_numpy(self.Rs).cuda()
            self._dev = d
        return self._dev

    def run(self, x16: np.ndarray, k: int, ws: dd.Workspace, idx: np.ndarray | None = None):
        """HIP path through the C ABI; returns (y fp16 numpy, idx int32 numpy, xsel fp16 numpy)."""
        d = self.device()
        xd = torch.from_numpy(x16).cuda()
        y = torch.full((self.N,), float("nan"), dtype=torch.float16, device="cuda")
        if idx is None:
            dd.decdec_gemv(self.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], k, y, ws)
            torch.cuda.synchronize()
            if k == 0:
                return y.cpu().numpy(), np.zeros(0, np.int32), np.zeros(0, np.float16)
            idx_h, xs_h = ws.read_selection(k)
            return y.cpu().numpy(), idx_h, xs_h
        idx_t = torch.from_numpy(np.ascontiguousarray(idx, np.int32)).cuda()
        xs_t = torch.from_numpy(np.ascontiguousarray(x16[idx])).cuda()
        dd.decdec_gemv_idx(self.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], d["Rs"], len(idx), idx_t, xs_t, y, ws)
        torch.cuda.synchronize()
        return y.cpu().numpy(), idx, x16[idx]

    def reference(self, x16: np.ndarray, k: int):
        sc = oracle.topk_abs(x16, k)
        return oracle.compensated_gemv(self.W_hat, x16, self.R_real, sc), sc


def assert_parity(y, y_ref, idx, sc, tol=TOL_Y, what=""):
    assert np.array_equal(idx, sc), f"{what}: selected channels differ from the oracle"
    err = oracle.error_metric(y.astype(np.float64), y_ref)
    assert np.all(np.isfinite(y.astype(np.float64))), what
    assert err <= tol, f"{what}: relative error {err:.3e} > {tol}"
    return err
