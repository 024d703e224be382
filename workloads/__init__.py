"""Seeded synthetic inputs for the DecDEC decode-step hot path.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no quantiser, no selection, no GEMV): both the CPU oracle's
tests and the HIP path's tests/benchmark take their raw inputs from here, and
neither of those two imports the other.

The inputs stand in for the workloads the paper measures on (linear layers of
Llama-3-8B / Llama-3-70B at batch 1, Section 5.1 and 5.5): only the layer
shapes are taken from those models; weights and activations are synthetic.

Orientation follows the paper (Section 3.1-3.2): a weight matrix is
d_in x d_out = K x N, a row is an input channel, a column an output channel.
"""
from __future__ import annotations

import numpy as np

ROOT_SEED = (2412, 20185)

# (name, K, N, name of the activation vector the GEMV consumes)
LLAMA3_8B_LAYER = (
    ("q", 4096, 4096, "attn_in"),
    ("k", 4096, 1024, "attn_in"),
    ("v", 4096, 1024, "attn_in"),
    ("o", 4096, 4096, "o_in"),
    ("gate", 4096, 14336, "mlp_in"),
    ("up", 4096, 14336, "mlp_in"),
    ("down", 14336, 4096, "down_in"),
)
LLAMA3_70B_LAYER = (
    ("q", 8192, 8192, "attn_in"),
    ("k", 8192, 1024, "attn_in"),
    ("v", 8192, 1024, "attn_in"),
    ("o", 8192, 8192, "o_in"),
    ("gate", 8192, 28672, "mlp_in"),
    ("up", 8192, 28672, "mlp_in"),
    ("down", 28672, 8192, "down_in"),
)
_INPUT_IDS = {"attn_in": 0, "o_in": 1, "mlp_in": 2, "down_in": 3}
_GEMV_IDS = {n: i for i, (n, _, _, _) in enumerate(LLAMA3_8B_LAYER)}


def _rng(*tags: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(ROOT_SEED) + [int(t) for t in tags])))


def k_for_fraction(K: int, frac: float) -> int:
    """Number of salient channels for a fraction of K (rounded down; the
    paper's example: 10 % of 14336 channels is 1433, Section 4.3)."""
    return int(np.floor(frac * K + 1e-9))


def k_for_kchunk(K: int, k_chunk: int) -> int:
    """k for k_chunk channels per 1024 input channels (Section 4.3/4.4)."""
    return (K // 1024) * int(k_chunk) if K % 1024 == 0 else int(K * k_chunk // 1024)


def weights(cfg: int, layer: int, gemv: str | int, K: int, N: int, sigma: float = 0.02) -> np.ndarray:
    """fp32 W[K][N] ~ N(0, sigma^2)."""
    gid = _GEMV_IDS[gemv] if isinstance(gemv, str) else int(gemv)
    g = _rng(cfg, layer, gid, 0)
    w = g.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(sigma)
    return w


def _to_f16(v: np.ndarray) -> np.ndarray:
    return np.clip(v, -65504.0, 65504.0).astype(np.float16)


def x_gauss_outliers(cfg: int, layer: int, which: str | int, step: int, K: int,
                     n_out: int | None = None, lo: float = 10.0, hi: float = 50.0) -> np.ndarray:
    """fp16 x[K] ~ N(0,1) with n_out (default floor(0.5 % K)) channels at fresh
    random positions multiplied by U(lo, hi)."""
    wid = _INPUT_IDS[which] if isinstance(which, str) else int(which)
    g = _rng(cfg, layer, 100 + wid, step)
    x = g.standard_normal(K)
    if n_out is None:
        n_out = int(np.floor(0.005 * K))
    if n_out > 0:
        pos = g.choice(K, size=n_out, replace=False)
        x[pos] *= g.uniform(lo, hi, size=n_out)
    return _to_f16(x)


def x_student_t(cfg: int, layer: int, which: str | int, step: int, K: int, nu: float = 3.0,
                outlier_frac: float = 0.0, outlier_mult: float = 30.0) -> np.ndarray:
    """fp16 x[K] ~ Student-t(nu); optionally floor(outlier_frac*K) channels at
    fresh random positions multiplied by outlier_mult."""
    wid = _INPUT_IDS[which] if isinstance(which, str) else int(which)
    g = _rng(cfg, layer, 200 + wid, step)
    x = g.standard_t(nu, size=K)
    n_out = int(np.floor(outlier_frac * K))
    if n_out > 0:
        pos = g.choice(K, size=n_out, replace=False)
        x[pos] *= outlier_mult
    return _to_f16(x)


def config1():
    """Single linear 1024x1024, 4-bit, k=32, x ~ N(0,1) with 10 channels x20."""
    K = N = 1024
    g = _rng(1, 0, 100, 0)
    x = g.standard_normal(K)
    pos = g.choice(K, size=10, replace=False)
    x[pos] *= 20.0
    return dict(K=K, N=N, bits=4, k=32, W=weights(1, 0, 0, K, N), x=_to_f16(x))
