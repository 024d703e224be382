"""GPU parity of the device quantiser: codes, scales, zero points and the fp16
residual must equal the oracle's bit for bit (every decision is one IEEE fp32
operation on both sides)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from paper_2412_20185_amd.layer import UniformLinear

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("K,N", [(1024, 1024), (384, 192), (4096, 1024)])
def test_quantiser_matches_oracle_bit_for_bit(bits, K, N):
    W = workloads.weights(70 + bits, 0, 0, K, N)
    W[128:256, 3] = 0.0125          # constant group: scale 0 -> 1
    W[0:128, 5] *= 1e-4             # tiny range: subnormal fp16 scale
    lin = UniformLinear(W, bits)
    codes, s, z = oracle.quantize_uniform(W, bits)
    assert np.array_equal(lin.scales.cpu().numpy().view(np.uint16), s.view(np.uint16))
    assert np.array_equal(lin.zeros.cpu().numpy().view(np.uint16), z.view(np.uint16))
    packed = lin.Wq.cpu().numpy()
    assert np.array_equal(dd.decdec_unpack_weights(lin.desc, packed), codes)
    assert np.array_equal(packed, dd.decdec_pack_weights(lin.desc, codes))
    R = oracle.residual_fp16(W, oracle.dequantize_uniform(codes, s, z))
    assert np.array_equal(lin.R.numpy().view(np.uint16), R.view(np.uint16))
