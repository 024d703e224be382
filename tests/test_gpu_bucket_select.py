"""GPU parity of decdec_select_bucket (the paper's approximate Top-K, Section
4.3) against oracle.topk_bucket: bit-exact indices, then the compensated GEMV
driven by that selection against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd
from helpers import Problem, assert_parity

pytestmark = pytest.mark.gpu


def run_bucket(x16, k_chunk, b0, b15):
    K = len(x16)
    n = k_chunk * K // 1024
    xd = torch.from_numpy(x16).cuda()
    idx = torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")
    xs = torch.zeros((max(n, 1),), dtype=torch.float16, device="cuda")
    dd.decdec_select_bucket(xd, K, k_chunk, b0, b15, idx, xs)
    torch.cuda.synchronize()
    return idx.cpu().numpy()[:n], xs.cpu().numpy()[:n]


def cases():
    g = np.random.default_rng(12)
    yield "outliers_4096", workloads.x_gauss_outliers(3, 0, "attn_in", 0, 4096), None
    yield "outliers_14336", workloads.x_gauss_outliers(3, 0, "down_in", 1, 14336), None
    yield "student_t_28672", workloads.x_student_t(4, 0, "down_in", 0, 28672), None
    yield "all_equal", np.full(2048, 0.75, np.float16), (4.0, 1.0)
    yield "few_values", g.integers(-3, 4, size=4096).astype(np.float16), (3.0, 2.0)
    yield "degenerate_b0_eq_b15", g.standard_normal(1024).astype(np.float16), (1.5, 1.5)
    yield "b15_zero", g.standard_normal(1024).astype(np.float16), (2.0, 0.0)
    sp = g.standard_normal(1024).astype(np.float16)
    sp[[3, 500]] = np.inf
    sp[7] = np.nan
    sp[9] = -0.0
    yield "inf_nan_zero", sp, (3.0, 1.0)
    on_edges = np.tile(np.concatenate([oracle.bucket_boundaries(8.0, 2.0), [0.0]]), 32).astype(np.float16)
    yield "values_on_boundaries", on_edges, (8.0, 2.0)


@pytest.mark.parametrize("name,x,bounds", list(cases()), ids=[c[0] for c in cases()])
def test_bucket_select_matches_oracle(name, x, bounds):
    K = len(x)
    for k_chunk in (1, 8, 20, 64, 367, 1024):
        if bounds is None:
            X = np.stack([np.roll(x, 17 * (s + 1)) for s in range(4)])
            b0, b15 = oracle.calibrate_boundaries(X, max(1, k_chunk * K // 1024))
        else:
            b0, b15 = bounds
        idx, xs = run_bucket(x, k_chunk, float(b0), float(b15))
        want = oracle.topk_bucket(x, k_chunk, b0, b15)
        assert np.array_equal(idx, want), (name, k_chunk)
        assert np.array_equal(xs.view(np.uint16), x[want].view(np.uint16)), (name, k_chunk)


def test_compensated_gemv_with_the_approximate_selection():
    """Selection by decdec_select_bucket, fed to decdec_gemv_idx: y against the oracle
    evaluated on the oracle's approximate selection; recall against the exact Top-K."""
    K, N, k_chunk = 4096, 1024, 32
    ws = dd.Workspace(K, N, K)
    p = Problem(workloads.weights(66, 0, 0, K, N), 3)
    d = p.device()
    X = np.stack([workloads.x_gauss_outliers(66, 0, 0, 100 + s, K) for s in range(16)])
    b0, b15 = oracle.calibrate_boundaries(X, k_chunk * K // 1024)
    k = k_chunk * K // 1024
    recalls = []
    for step in range(4):
        x = workloads.x_gauss_outliers(66, 0, 0, step, K)
        xd = torch.from_numpy(x).cuda()
        idx = torch.empty(k, dtype=torch.int32, device="cuda")
        xs = torch.empty(k, dtype=torch.float16, device="cuda")
        y = torch.empty(N, dtype=torch.float16, device="cuda")
        dd.decdec_select_bucket(xd, K, k_chunk, float(b0), float(b15), idx, xs)
        dd.decdec_gemv_idx(p.desc, xd, d["Wq"], d["scales"], d["zl"], d["R"], None, k, idx, xs, y, ws)
        torch.cuda.synchronize()
        sc = oracle.topk_bucket(x, k_chunk, b0, b15)
        y_ref = oracle.compensated_gemv(p.W_hat, x, p.R_real, sc)
        assert_parity(y.cpu().numpy(), y_ref, idx.cpu().numpy(), sc, what=f"approx select step {step}")
        recalls.append(oracle.recall(sc, oracle.topk_abs(x, k)))
    print(f"recall of the approximate selector against the exact Top-K: {np.mean(recalls):.3f}")
    assert np.mean(recalls) > 0.6
    ws.close()
