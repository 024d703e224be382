"""Step 1 of dynamic error compensation: the salient-channel list.

Test infrastructure only (see oracle/__init__.py).
"""
from __future__ import annotations

import numpy as np


def magnitude_keys(x16: np.ndarray) -> np.ndarray:
    """|x| as an ordered integer: the fp16 bit pattern with the sign cleared.

    For every non-NaN fp16 value this orders exactly like |x| (+0 and -0 both
    give 0, infinity is above every finite value); NaN patterns sort above
    infinity, which makes the selection total and deterministic on any input.
    """
    x16 = np.ascontiguousarray(x16, dtype=np.float16)
    return (x16.view(np.uint16) & np.uint16(0x7FFF)).astype(np.int32)


def topk_abs(x16: np.ndarray, k: int) -> np.ndarray:
    """sc_indices: the k channels with the largest |x| (Section 4.1 step 1,
    the exact Top-K of Section 5.2), a tie at the cut going to the lower
    index; returned in ascending index order as int32."""
    key = magnitude_keys(x16)
    K = key.shape[0]
    if not 0 <= k <= K:
        raise ValueError("k out of range")
    order = np.argsort(-key, kind="stable")      # descending key, ascending index among equals
    return np.sort(order[:k]).astype(np.int32)
