"""GPU parity of decdec_select_topk against oracle.topk_abs: bit-exact indices,
including ties at the cut, signed zeros, all-equal inputs and every k edge."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_2412_20185_amd as dd

pytestmark = pytest.mark.gpu


def run_select(x16, k):
    K = len(x16)
    xd = torch.from_numpy(x16).cuda()
    idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
    xs = torch.zeros((max(k, 1),), dtype=torch.float16, device="cuda")
    dd.decdec_select_topk(xd, K, k, idx, xs)
    torch.cuda.synchronize()
    return idx.cpu().numpy()[:k], xs.cpu().numpy()[:k]


def cases():
    g = np.random.default_rng(3)
    yield "gauss4096", g.standard_normal(4096).astype(np.float16)
    yield "all_equal", np.full(1024, -1.5, np.float16)
    yield "few_values", g.integers(-3, 4, size=14336).astype(np.float16)
    z = np.zeros(2048, np.float16)
    z[::2] = -0.0
    z[5] = 1e-7
    yield "zeros_signed", z
    yield "student_t_28672", workloads.x_student_t(4, 0, "down_in", 0, 28672)
    yield "outliers_14336", workloads.x_gauss_outliers(2, 0, "down_in", 0, 14336)
    yield "ragged_K_1000", g.standard_normal(1000).astype(np.float16)
    yield "tiny_K_8", g.standard_normal(8).astype(np.float16)
    yield "max_K_65536", g.standard_t(3, size=65536).astype(np.float16)
    big = g.standard_normal(512).astype(np.float16)
    big[[3, 77]] = np.inf
    big[100] = -np.inf
    yield "infinities", big
    nans = g.standard_normal(1024).astype(np.float16)
    nans.view(np.uint16)[[5, 600]] = [0x7E00, 0xFC01]      # quiet and signalling patterns: keys above infinity
    nans[7] = np.inf
    yield "nans", nans


@pytest.mark.parametrize("name,x", list(cases()), ids=[c[0] for c in cases()])
def test_select_matches_oracle(name, x):
    K = len(x)
    ks = sorted({0, 1, 2, K // 100 + 1, workloads.k_for_fraction(K, 0.02), K // 2, K - 1, K})
    for k in ks:
        if k > K:
            continue
        idx, xs = run_select(x, k)
        sc = oracle.topk_abs(x, k)
        assert np.array_equal(idx, sc), (name, k)
        assert np.array_equal(xs.view(np.uint16), x[sc].view(np.uint16)), (name, k)


def test_select_redrawn_outliers_many_steps():
    """Config 3/5 style: outlier positions redrawn every step."""
    for step in range(32):
        for K, which in ((4096, "attn_in"), (14336, "down_in")):
            x = workloads.x_gauss_outliers(3, 0, which, step, K)
            k = workloads.k_for_kchunk(K, 32)
            idx, _ = run_select(x, k)
            assert np.array_equal(idx, oracle.topk_abs(x, k)), (step, K)
