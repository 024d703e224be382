"""Steps 2-4: the compensated GEMV, written out as its definition in fp64.

Test infrastructure only (see oracle/__init__.py).
"""
from __future__ import annotations

import numpy as np


def compensated_gemv(W_hat: np.ndarray, x16: np.ndarray, R_hat: np.ndarray | None, sc: np.ndarray) -> np.ndarray:
    """o = W_hat^T x + R_hat[sc, :]^T x[sc]   (Section 3.1, Section 4.1).

    W_hat: fp64 [K][N] de-quantised weights; x16: fp16 [K]; R_hat: [K][N]
    stored residual as real numbers (any float dtype); sc: selected channels.
    Returns fp64 [N].
    """
    x = np.asarray(x16, dtype=np.float64)
    o_b = np.asarray(W_hat, dtype=np.float64).T @ x
    sc = np.asarray(sc, dtype=np.intp)
    if sc.size == 0:
        return o_b
    o_dec = np.asarray(R_hat[sc, :], dtype=np.float64).T @ x[sc]
    return o_b + o_dec


def compensated_gemv_columns(dequant_column, x16, R_hat_rows, sc, cols) -> np.ndarray:
    """The same result for a few output columns only, one at a time.

    dequant_column(n) -> fp64 [K] column n of W_hat; R_hat_rows(sc, n) -> fp64
    [len(sc)] entries R_hat[sc, n].  Used where the full matrix is too large
    to de-quantise in fp64 at once.
    """
    x = np.asarray(x16, dtype=np.float64)
    sc = np.asarray(sc, dtype=np.intp)
    out = np.empty(len(cols), dtype=np.float64)
    for i, n in enumerate(cols):
        o = float(np.dot(dequant_column(int(n)), x))
        if sc.size:
            o += float(np.dot(R_hat_rows(sc, int(n)), x[sc]))
        out[i] = o
    return out


def error_metric(y, y_ref, rms=None) -> float:
    """max_n |y - y_ref| / max(|y_ref[n]|, 0.01 * rms(y_ref)).

    A plain element-wise relative error with a floor on the denominator so
    that outputs which happen to cancel to nearly zero do not dominate.
    """
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    if y_ref.size == 0:
        return 0.0
    if rms is None:
        rms = float(np.sqrt(np.mean(y_ref ** 2)))
    den = np.maximum(np.abs(y_ref), 0.01 * rms)
    den = np.where(den == 0, 1.0, den)
    return float(np.max(np.abs(y - y_ref) / den))
