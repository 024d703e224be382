"""Offline steps of the oracle: base quantisers, de-quantisers, residuals.

Test infrastructure only (see oracle/__init__.py).

Layouts (all row-major NumPy arrays, orientation of Section 3.1-3.2: K x N,
row = input channel, column = output channel):
  W       float32 [K][N]
  codes   uint8   [K][N]      one code per byte
  scales  float16 [K/128][N]  (uniform) one per column per group of 128 rows
  zeros   float16 [K/128][N]  integer-valued zero points
  lut     float16 [N][8]      (non-uniform) one ascending codebook per column
  R       float16 [K][N]      residual, or
  Rq      int8    [K][N] in [-7, 7] with Rs float16 [N]   (Section 4.2)
"""
from __future__ import annotations

import numpy as np

GROUP = 128


def quantize_uniform(W: np.ndarray, bits: int, group: int = GROUP):
    """Uniform asymmetric min/max quantiser, one (scale, zero) per output
    column per `group` consecutive input channels.

    The paper takes its uniform base quantiser from third-party work
    (Section 5.2 methodology) and prints no formula; this is the build's
    reading.  Every decision is taken in IEEE fp32 (one rounding per
    operation, no fusion) so that an fp32 device implementation can reproduce
    the integer codes exactly:
        s  = fp16(fp32(hi - lo) / (2^b - 1)),  s = 1 if that is 0
        z  = clip(rint(-lo / s), 0, 2^b - 1)      (stored as +0, never -0)
        q  = clip(rint(w / s) + z, 0, 2^b - 1)
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    K, N = W.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    qmax = np.float32(2 ** bits - 1)
    Wg = W.reshape(K // group, group, N)
    lo = Wg.min(axis=1)
    hi = Wg.max(axis=1)
    s32 = ((hi - lo).astype(np.float32) / qmax).astype(np.float32)
    s = s32.astype(np.float16)
    s[s == 0] = np.float16(1.0)
    sf = s.astype(np.float32)
    z = (np.clip(np.rint((-lo / sf).astype(np.float32)), 0, qmax) + np.float32(0)).astype(np.float32)  # +0: never -0
    q = np.rint((Wg / sf[:, None, :]).astype(np.float32)) + z[:, None, :]
    q = np.clip(q, 0, qmax)
    return q.astype(np.uint8).reshape(K, N), s, z.astype(np.float16)


def dequantize_uniform(codes, scales, zeros, group: int = GROUP) -> np.ndarray:
    """W_hat[k][n] = s[k/group][n] * (q[k][n] - z[k/group][n]) in fp64."""
    s = np.repeat(np.asarray(scales, dtype=np.float64), group, axis=0)
    z = np.repeat(np.asarray(zeros, dtype=np.float64), group, axis=0)
    return s * (np.asarray(codes, dtype=np.float64) - z)


def quantize_lut(W: np.ndarray, iters: int = 16, levels: int = 8, chunk: int = 256):
    """Non-uniform (clustering) quantiser: one `levels`-entry codebook per
    output column from plain 1-D Lloyd k-means over that column (fp64).

    Stands for the clustering-based non-uniform base quantiser the paper uses
    (Section 5.2 methodology) without its sensitivity weighting, which needs
    gradients of a real model.  Centroids start at the (i + 0.5)/levels
    quantiles, run `iters` Lloyd steps (an empty cluster keeps its centroid),
    are sorted, rounded to fp16, and every weight takes the nearest stored
    centroid (ties to the lower code).
    """
    W = np.asarray(W, dtype=np.float64)
    K, N = W.shape
    codes = np.empty((K, N), dtype=np.uint8)
    lut = np.empty((N, levels), dtype=np.float16)
    qs = (np.arange(levels) + 0.5) / levels
    for n0 in range(0, N, chunk):
        v = W[:, n0:n0 + chunk]                      # [K, c]
        c = np.quantile(v, qs, axis=0).T.copy()      # [c, levels]
        for _ in range(iters):
            a = np.abs(v[:, :, None] - c[None, :, :]).argmin(axis=2)   # [K, c]
            for j in range(levels):
                m = a == j
                cnt = m.sum(axis=0)
                sm = np.where(m, v, 0.0).sum(axis=0)
                c[:, j] = np.where(cnt > 0, sm / np.maximum(cnt, 1), c[:, j])
        c.sort(axis=1)
        l16 = c.astype(np.float16)
        lut[n0:n0 + chunk] = l16
        a = np.abs(v[:, :, None] - l16.astype(np.float64)[None, :, :]).argmin(axis=2)
        codes[:, n0:n0 + chunk] = a.astype(np.uint8)
    return codes, lut


def dequantize_lut(codes, lut) -> np.ndarray:
    """W_hat[k][n] = lut[n][codes[k][n]] in fp64."""
    codes = np.asarray(codes)
    K, N = codes.shape
    l = np.asarray(lut, dtype=np.float64)
    return l[np.arange(N)[None, :], codes.astype(np.intp)]


def residual_fp16(W, W_hat) -> np.ndarray:
    """R = fp16(W - W_hat), round to nearest even, subnormals kept
    (Section 3.1: R is the residual between original and quantised weights)."""
    return (np.asarray(W, dtype=np.float64) - np.asarray(W_hat, dtype=np.float64)).astype(np.float16)


DEFAULT_ALPHAS = np.round(np.arange(30, 101) / 100.0, 2)


def quantize_residual_sym(R, bits, alphas=DEFAULT_ALPHAS):
    """b-bit symmetric residual quantiser, one scale per output column:
    Q_i(r) = clip(round_to_int(r / S_i), -qmax, qmax) with
    qmax = 2^(b-1) - 1, S_i found by grid search for the least squared error
    of column i.  b = 4 (qmax 7) is the quantiser of Section 4.2; b = 2
    (codes -1, 0, 1) and b = 8 (qmax 127) are the other integer widths of the
    residual bit-width study (Table 2).

    Reading of what the paper leaves open: round_to_int is round-half-even;
    the grid is S = fp16(alpha * max|r| / qmax) for alpha in `alphas`
    (0.30 ... 1.00 step 0.01); ties keep the larger alpha; an all-zero column
    gets S = 1; the 2- and 8-bit quantisers (not written out in the paper)
    are the same formula with their own qmax.
    """
    if bits not in (2, 4, 8):
        raise ValueError("bits must be 2, 4 or 8")
    qmax = float(2 ** (bits - 1) - 1)
    R = np.asarray(R, dtype=np.float64)
    K, N = R.shape
    m = np.abs(R).max(axis=0)
    best_err = np.full(N, np.inf)
    best_S = np.ones(N, dtype=np.float16)
    for a in alphas:
        S = (a * m / qmax).astype(np.float16)
        S[S == 0] = np.float16(1.0)
        Sd = S.astype(np.float64)
        q = np.clip(np.rint(R / Sd), -qmax, qmax)
        err = ((R - Sd * q) ** 2).sum(axis=0)
        take = err <= best_err
        best_err = np.where(take, err, best_err)
        best_S = np.where(take, S, best_S)
    Sd = best_S.astype(np.float64)
    q = np.clip(np.rint(R / Sd), -qmax, qmax).astype(np.int8)
    return q, best_S


def quantize_residual_int4(R, alphas=DEFAULT_ALPHAS):
    """The 4-bit residual quantiser of Section 4.2 (codes in [-7, 7])."""
    return quantize_residual_sym(R, 4, alphas)


def dequantize_residual_int4(Rq, Rs) -> np.ndarray:
    """R_hat[k][n] = S[n] * q[k][n] in fp64."""
    return np.asarray(Rq, dtype=np.float64) * np.asarray(Rs, dtype=np.float64)[None, :]
