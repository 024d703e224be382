"""CPU oracle for the DecDEC decode-step hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow NumPy code in fp64 (integer decisions of the offline quantisers in
the precision stated per function).  It exists to check the HIP kernels and is
imported only by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg
of bench.py.  It shares no code with the HIP path and never imports it; the
product path never imports this package.

What it computes (DecDEC, Section 3.1 and Section 4.1):

    o = W_hat x  +  R_hat[sc_indices, :]^T  x[sc_indices]

with W_hat the de-quantised weights (d_in x d_out = K x N, rows are input
channels), R_hat the stored residual W - W_hat kept in CPU memory, and
sc_indices the k input channels with the largest |x| this step (the exact
Top-K arm of Section 5.2, ties resolved toward the lower index).

Pinned by tests/test_oracle_*.py and tests/test_paper_values.py against the
numbers the paper prints, brute force with exact rationals,
closed forms (weights on the quantisation grid), the k = 0 and k = K
invariants, scaling laws and a planted-mistake check per function.
Functions without an external pin: none ("parity unpinned" applies to nothing
here); the base quantisers follow this build's reading of an unspecified
third-party step and are pinned only as to their stated definition.
"""
from .quantize import (  # noqa: F401
    GROUP, quantize_uniform, dequantize_uniform, quantize_lut, dequantize_lut,
    residual_fp16, quantize_residual_sym, quantize_residual_int4, dequantize_residual_int4,
)
from .select import topk_abs, magnitude_keys  # noqa: F401
from .bucket_select import (  # noqa: F401
    bucket_boundaries, bucket_index, topk_bucket, calibrate_boundaries, recall,
)
from .gemv import compensated_gemv, compensated_gemv_columns, error_metric  # noqa: F401
