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


def _residual_f32_reference(W, W_hat):
    """fp32 of W - W_hat (the difference itself is exact in fp64 for these magnitudes)."""
    return (W.astype(np.float64) - W_hat).astype(np.float32)


@pytest.mark.parametrize("wfmt,bits", [("uniform", 3), ("uniform", 4), ("lut", 3)])
def test_residual_f32_of_packed_weights(wfmt, bits):
    """R = W - W_hat from the packed weights, whatever base quantiser produced them."""
    K, N = 640, 192
    W = workloads.weights(75, 0, 0, K, N)
    if wfmt == "uniform":
        codes, s, z = oracle.quantize_uniform(W, bits)
        W_hat = oracle.dequantize_uniform(codes, s, z)
        desc = dd.Desc(K, N, bits)
        s_d, zl_d = torch.from_numpy(s).cuda(), torch.from_numpy(z).cuda()
    else:
        codes, lut = oracle.quantize_lut(W, iters=2)
        W_hat = oracle.dequantize_lut(codes, lut)
        desc = dd.Desc(K, N, 3, dd.W_LUT_COL8)
        s_d, zl_d = None, torch.from_numpy(lut).cuda()
    Wq = torch.from_numpy(dd.decdec_pack_weights(desc, codes)).cuda()
    R = torch.full((K, N), float("nan"), dtype=torch.float32, device="cuda")
    dd.decdec_residual_f32(desc, torch.from_numpy(W).cuda(), Wq, s_d, zl_d, R)
    torch.cuda.synchronize()
    assert np.array_equal(R.cpu().numpy().view(np.uint32), _residual_f32_reference(W, W_hat).view(np.uint32))


@pytest.mark.parametrize("rbits", [2, 4, 8])
@pytest.mark.parametrize("K,N", [(1024, 512), (384, 192)])
def test_residual_quantiser_matches_oracle_bit_for_bit(rbits, K, N):
    """Section 4.2's quantiser and its 2- and 8-bit variants: scales and codes equal the oracle's.
    Both sides decide in fp64, one IEEE operation per step, column errors summed in ascending k."""
    g = np.random.default_rng([76, rbits, K])
    R32 = (g.standard_normal((K, N)) * 2e-3).astype(np.float32)
    R32[:, 3] = 0.0                       # all-zero column: S = 1
    R32[:, 5] *= 1e-5                     # subnormal fp16 scales
    R32[7, 9] = 0.05                      # one outlier: the search clips it
    q_ref, S_ref = oracle.quantize_residual_sym(R32.astype(np.float64), rbits)
    codes = torch.zeros((K, N * rbits // 8), dtype=torch.uint8, pin_memory=True)
    S = torch.zeros(N, dtype=torch.float16, device="cuda")
    dd.decdec_quantize_residual(K, N, rbits, torch.from_numpy(R32).cuda(), codes, S)
    torch.cuda.synchronize()
    assert np.array_equal(S.cpu().numpy().view(np.uint16), S_ref.view(np.uint16))
    assert np.array_equal(codes.numpy(), dd.decdec_pack_residual_int(q_ref, rbits))


@pytest.mark.parametrize("rbits", [4, 2, 8])
def test_uniform_linear_with_integer_residuals_end_to_end(rbits):
    """Device-prepared layer (quantiser, fp32 residual, residual quantiser) through the hot path,
    against the oracle run on the oracle's own artefacts of the same W."""
    K, N, bits, k = 1024, 512, 3, 40
    W = workloads.weights(77, 0, 0, K, N)
    lin = UniformLinear(W, bits, rbits=rbits)
    codes, s, z = oracle.quantize_uniform(W, bits)
    W_hat = oracle.dequantize_uniform(codes, s, z)
    q_ref, S_ref = oracle.quantize_residual_sym(_residual_f32_reference(W, W_hat).astype(np.float64), rbits)
    assert np.array_equal(lin.R.numpy(), dd.decdec_pack_residual_int(q_ref, rbits))
    assert np.array_equal(lin.R_scales.cpu().numpy().view(np.uint16), S_ref.view(np.uint16))
    x = workloads.x_gauss_outliers(77, 0, 0, 0, K)
    sc = oracle.topk_abs(x, k)
    y_ref = oracle.compensated_gemv(W_hat, x, oracle.dequantize_residual_int4(q_ref, S_ref), sc)
    ws = dd.Workspace(K, N, k)
    try:
        y = torch.empty(N, dtype=torch.float16, device="cuda")
        lin.gemv(torch.from_numpy(x).cuda(), k, y, ws)
        torch.cuda.synchronize()
        assert np.array_equal(ws.read_selection(k)[0], sc)
        assert oracle.error_metric(y.cpu().numpy().astype(np.float64), y_ref) <= 2e-3
    finally:
        ws.close()
