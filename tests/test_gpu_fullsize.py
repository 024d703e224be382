"""GPU parity at the full sizes of the BASELINE configs, in the launch
configuration bench.py times.  Llama-3-8B shapes: the oracle quantises and
checks every output.  Llama-3-70B shapes (235 M weights): stored parameters
are drawn directly (random codes, a random ascending codebook per column, small
random fp16 residuals) and the oracle computes sampled output columns one by
one; the selection is checked in full."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity, TOL_Y

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ws():
    w = dd.Workspace(28672, 28672, 2048)
    yield w
    w.close()


@pytest.mark.parametrize("name", ["q", "k", "gate", "down"])
@pytest.mark.parametrize("bits", [3, 4])
def test_llama3_8b_shapes_full_check(ws, name, bits):
    """Configs 2 (3-bit, k = 2 %) and 3 (4-bit, k_chunk sweep incl. 0 and 128 per 1024)."""
    _, K, N, which = next(s for s in workloads.LLAMA3_8B_LAYER if s[0] == name)
    p = Problem(workloads.weights(2, 0, name, K, N), bits)
    ks = [workloads.k_for_fraction(K, 0.02)] if bits == 3 else [0, workloads.k_for_kchunk(K, 8),
                                                                workloads.k_for_kchunk(K, 128)]
    for step, k in enumerate(ks):
        x = workloads.x_gauss_outliers(2, 0, which, step, K)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        err = assert_parity(y, y_ref, idx, sc, what=f"8B {name} b{bits} k={k}")
        print(f"8B {name} {K}x{N} b{bits} k={k}: rel err {err:.2e}")


def test_llama3_8b_down_int4_residuals(ws):
    """Config 5: 3-bit weights, 4-bit per-column-scaled residuals, k_chunk = 15 (k = 210)."""
    K, N = 14336, 4096
    p = Problem(workloads.weights(5, 0, "down", K, N), 3, rfmt="int4", alphas=oracle.quantize.DEFAULT_ALPHAS[::10])
    k = workloads.k_for_kchunk(K, 15)
    assert k == 210
    for step in range(2):
        x = workloads.x_student_t(5, 0, "down_in", step, K, outlier_frac=0.005, outlier_mult=30.0)
        y_ref, sc = p.reference(x, k)
        y, idx, _ = p.run(x, k, ws)
        assert_parity(y, y_ref, idx, sc, what="8B down int4")


@pytest.mark.parametrize("K,N", [(8192, 28672), (28672, 8192), (8192, 1024)])
def test_llama3_70b_lut_shapes_sampled(ws, K, N):
    """Config 4: 3-bit codebook weights, Student-t activations, k = 1 % of K."""
    g = np.random.default_rng([4, K, N])
    codes = g.integers(0, 8, size=(K, N), dtype=np.uint8)
    lut = np.sort(g.standard_normal((N, 8)) * 0.02, axis=1).astype(np.float16)
    R = (g.standard_normal((K, N), dtype=np.float32) * np.float32(0.003)).astype(np.float16)
    desc = dd.Desc(K, N, 3, dd.W_LUT_COL8, dd.R_FP16)
    Wq = torch.from_numpy(dd.decdec_pack_weights(desc, codes)).cuda()
    lut_d = torch.from_numpy(lut).cuda()
    R_p = torch.from_numpy(R).pin_memory()
    k = workloads.k_for_fraction(K, 0.01)
    x = workloads.x_student_t(4, 0, "down_in" if K > N else "mlp_in", 0, K)
    y = torch.empty(N, dtype=torch.float16, device="cuda")
    dd.decdec_gemv(desc, torch.from_numpy(x).cuda(), Wq, None, lut_d, R_p, None, k, y, ws)
    torch.cuda.synchronize()
    idx, xsel = ws.read_selection(k)
    sc = oracle.topk_abs(x, k)
    assert np.array_equal(idx, sc)
    assert np.array_equal(xsel.view(np.uint16), x[sc].view(np.uint16))
    cols = np.sort(g.choice(N, 96, replace=False))
    cols[0], cols[-1] = 0, N - 1
    lut64 = lut.astype(np.float64)
    y_ref = oracle.compensated_gemv_columns(lambda n: lut64[n][codes[:, n]], x,
                                            lambda s, n: R[s, n].astype(np.float64), sc, cols)
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    err = oracle.error_metric(y.cpu().numpy().astype(np.float64)[cols], y_ref, rms=rms)
    assert np.all(np.isfinite(y.cpu().numpy().astype(np.float64)))
    assert err <= TOL_Y, err
    print(f"70B {K}x{N} lut3 k={k}: rel err on 96 sampled columns {err:.2e}")
