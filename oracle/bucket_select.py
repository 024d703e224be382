"""The paper's fast approximate Top-K (DecDEC Section 4.3, "Fast Approximate
Top-K for Channel Selection"), as a plain CPU reference.

Test infrastructure only (see oracle/__init__.py).

x is cut into contiguous chunks of 1024 channels; every chunk contributes
k_chunk channels.  Inside a chunk the magnitudes are scattered into 32 buckets
with boundaries b_0 > b_1 > ... > b_30 derived from two calibrated values:
    b_i = b_0 - i (b_0 - b_15) / 15        for 0 <= i <= 15   (above b_15)
    b_i = b_15 (31 - i) / 16               for 15 <= i <= 30  (below b_15)
bucket 0 holds |x| >= b_0, bucket i (1..30) holds b_i <= |x| < b_(i-1), bucket 31
holds |x| < b_30.  Channels are gathered from bucket 0 upwards until k_chunk
are found; the bucket that overflows is filled "randomly" in the paper.

Readings where the paper leaves room:
  * the overflowing bucket is filled with its lowest channel indices (a
    deterministic stand-in for the paper's random choice, matching the tie rule
    of the exact selector);
  * the bucket of a value is computed in fp32 exactly as written in
    bucket_index() so that a device implementation can reproduce it bit for bit
    (a value within rounding of a boundary may land on either side of it
    compared with boundaries evaluated in exact arithmetic);
  * the output is the concatenation over chunks, each chunk's channels in
    ascending index order.
"""
from __future__ import annotations

import numpy as np

CHUNK = 1024


def bucket_boundaries(b0: float, b15: float) -> np.ndarray:
    """b_0 ... b_30 in fp64, for documentation and tests."""
    b0, b15 = float(b0), float(b15)
    hi = [b0 - i * (b0 - b15) / 15.0 for i in range(16)]
    lo = [b15 * (31 - i) / 16.0 for i in range(16, 31)]
    return np.array(hi + lo)


def bucket_index(x16: np.ndarray, b0, b15) -> np.ndarray:
    """Bucket number 0..31 of every element; every operation is one fp32 operation."""
    f32 = np.float32
    a = np.abs(np.asarray(x16, dtype=np.float16).astype(f32))
    b0, b15 = f32(b0), f32(b15)
    w_hi = f32(f32(b0 - b15) / f32(15.0))
    w_lo = f32(b15 / f32(16.0))
    with np.errstate(divide="ignore", invalid="ignore"):
        t_hi = np.ceil((f32(b0) - a).astype(f32) / w_hi) if w_hi > 0 else np.ones_like(a)
        t_lo = np.floor(a / w_lo) if w_lo > 0 else np.zeros_like(a)
    hi = np.clip(np.nan_to_num(t_hi, nan=1.0, posinf=15.0, neginf=1.0), 1, 15).astype(np.int32)
    lo = 31 - np.clip(np.nan_to_num(t_lo, nan=0.0, posinf=15.0), 0, 15).astype(np.int32)
    out = np.where(a >= b0, 0, np.where(a >= b15, hi, lo)).astype(np.int32)
    out[np.isnan(a)] = 0          # NaN ranks above everything, as in the exact selector
    return out


def topk_bucket(x16: np.ndarray, k_chunk: int, b0, b15) -> np.ndarray:
    """sc_indices of the approximate selector: k_chunk channels per 1024-chunk."""
    x16 = np.asarray(x16, dtype=np.float16)
    K = x16.shape[0]
    if K % CHUNK or not 0 <= k_chunk <= CHUNK:
        raise ValueError("K must be a multiple of 1024 and 0 <= k_chunk <= 1024")
    bucket = bucket_index(x16, b0, b15)
    out = []
    for c in range(K // CHUNK):
        b = bucket[c * CHUNK:(c + 1) * CHUNK]
        order = np.argsort(b, kind="stable")            # bucket ascending, index ascending inside a bucket
        out.append(np.sort(order[:k_chunk]) + c * CHUNK)
    return np.concatenate(out).astype(np.int32) if out else np.zeros(0, np.int32)


def calibrate_boundaries(X16: np.ndarray, k: int):
    """(b_0, b_15) from calibration vectors X [n][K] (Section 4.3): b_15 is the
    largest, over the vectors, of the k-th largest |x| of a vector; b_0 the
    largest |x| seen at all."""
    A = np.abs(np.asarray(X16, dtype=np.float16).astype(np.float32))
    if not 1 <= k <= A.shape[1]:
        raise ValueError("k out of range")
    kth = np.sort(A, axis=1)[:, A.shape[1] - k]
    return np.float32(A.max()), np.float32(kth.max())


def recall(selected: np.ndarray, reference: np.ndarray) -> float:
    """Share of the reference channels that the selection contains (Section 5.2)."""
    if len(reference) == 0:
        return 1.0
    return float(len(np.intersect1d(selected, reference))) / float(len(reference))
