"""Pins for the oracle of the paper's approximate Top-K (Section 4.3): scalar
brute force against the printed boundary rule, invariants, the case in which it
must coincide with the exact per-chunk Top-K, calibration, planted mistakes."""
import numpy as np
import pytest

import oracle
from oracle import bucket_select as bs


def brute_bucket(a: float, b0: float, b15: float) -> int:
    """Bucket by comparing with the 31 boundaries of Figure 9, in exact (fp64) arithmetic."""
    b = bs.bucket_boundaries(b0, b15)
    if a >= b[0]:
        return 0
    for i in range(1, 31):
        if b[i] <= a < b[i - 1]:
            return i
    return 31


def brute_select(x16, k_chunk, b0, b15):
    out = []
    for c in range(len(x16) // 1024):
        chunk = [abs(float(v)) for v in x16[c * 1024:(c + 1) * 1024]]
        buckets = [[] for _ in range(32)]
        for i, a in enumerate(chunk):
            buckets[brute_bucket(a, b0, b15)].append(i)          # scatter, index order inside a bucket
        got = []
        for b in range(32):                                      # gather from bucket 0 upwards
            room = k_chunk - len(got)
            got += buckets[b][:room]                             # an overflowing bucket gives its lowest indices
        out += [c * 1024 + i for i in sorted(got)]
    return out


def mid_bucket_values(g, n, b0, b15):
    """n magnitudes that sit well inside buckets (never within rounding of a boundary)."""
    b = bs.bucket_boundaries(b0, b15)
    edges = np.concatenate([[b0 * 1.5], b, [0.0]])               # bucket i lies between edges[i+1] and edges[i]
    which = g.integers(0, 32, size=n)
    frac = g.uniform(0.25, 0.75, size=n)
    v = edges[which + 1] + frac * (edges[which] - edges[which + 1])
    return (v * g.choice([-1.0, 1.0], size=n)).astype(np.float16), which


def check(selector):
    g = np.random.default_rng(5)
    b0, b15 = 8.0, 2.0
    x, which = mid_bucket_values(g, 3072, b0, b15)
    # fp16 rounding must not have moved a value across a boundary
    assert all(brute_bucket(abs(float(v)), b0, b15) == w for v, w in zip(x[:200], which[:200]))
    for k_chunk in (0, 1, 7, 32, 100, 1024):
        try:
            got = list(np.asarray(selector(x, k_chunk, b0, b15)).tolist())
        except Exception:
            return False
        if got != brute_select(x, k_chunk, b0, b15):
            return False
    return True


def test_matches_brute_force_and_planted_mistakes_fail():
    assert check(oracle.topk_bucket)

    def from_the_small_end(x, k_chunk, b0, b15):
        return oracle.topk_bucket(x, k_chunk, b0, b15)[::-1] if k_chunk == 0 else _variant(x, k_chunk, b0, b15, rev=True)

    def overflow_takes_high_indices(x, k_chunk, b0, b15):
        return _variant(x, k_chunk, b0, b15, high=True)

    def global_instead_of_per_chunk(x, k_chunk, b0, b15):
        b = oracle.bucket_index(x, b0, b15)
        order = np.argsort(b, kind="stable")
        return np.sort(order[:k_chunk * (len(x) // 1024)])

    def signed_values(x, k_chunk, b0, b15):
        return oracle.topk_bucket(np.maximum(x, np.float16(0)), k_chunk, b0, b15)

    for bad in (from_the_small_end, overflow_takes_high_indices, global_instead_of_per_chunk, signed_values):
        assert not check(bad), bad.__name__


def _variant(x, k_chunk, b0, b15, rev=False, high=False):
    b = oracle.bucket_index(x, b0, b15)
    out = []
    for c in range(len(x) // 1024):
        bb = b[c * 1024:(c + 1) * 1024].astype(np.int64)
        key = -bb if rev else bb
        idx = np.arange(1024)
        order = np.lexsort((-idx if high else idx, key))
        out.append(np.sort(order[:k_chunk]) + c * 1024)
    return np.concatenate(out)


def test_bucket_index_formula_against_boundaries_on_random_values():
    g = np.random.default_rng(6)
    b0, b15 = np.float32(37.5), np.float32(2.5234375)
    x = (g.standard_t(3, size=20000) * 2).astype(np.float16)
    got = oracle.bucket_index(x, b0, b15)
    b = bs.bucket_boundaries(b0, b15)
    a = np.abs(x.astype(np.float64))
    near = np.min(np.abs(a[:, None] - b[None, :]) / np.maximum(b[None, :], 1e-9), axis=1) < 1e-5
    want = np.array([brute_bucket(v, float(b0), float(b15)) for v in a])
    assert np.array_equal(got[~near], want[~near])
    assert np.all(np.abs(got[near] - want[near]) <= 1)           # at a boundary: either neighbour
    assert got.min() >= 0 and got.max() <= 31
    # special values: exact ends, zero, beyond b0, NaN
    sp = np.array([0.0, -0.0, float(b15), float(b0), 60000.0, np.inf, np.nan], np.float16)
    assert oracle.bucket_index(sp, b0, b15).tolist() == [31, 31, 15, 0, 0, 0, 0]


def test_invariants_and_agreement_with_exact_when_buckets_separate():
    g = np.random.default_rng(7)
    K, k_chunk = 4096, 24
    x = (g.standard_normal(K)).astype(np.float16)
    X = np.stack([(g.standard_normal(K)).astype(np.float16) for _ in range(16)])
    b0, b15 = oracle.calibrate_boundaries(X, k_chunk * K // 1024)
    sel = oracle.topk_bucket(x, k_chunk, b0, b15)
    assert len(sel) == k_chunk * 4 and np.all(np.diff(sel) > 0)
    bucket = oracle.bucket_index(x, b0, b15)
    for c in range(4):
        s = sel[(sel >= c * 1024) & (sel < (c + 1) * 1024)]
        assert len(s) == k_chunk
        rest = np.setdiff1d(np.arange(c * 1024, (c + 1) * 1024), s)
        cut = bucket[s].max()
        assert cut <= bucket[rest].min()
        tie_in, tie_out = s[bucket[s] == cut], rest[bucket[rest] == cut]
        if len(tie_out):
            assert tie_in.max() < tie_out.min()
    # one distinct bucket per magnitude level: the approximation is exact per chunk
    levels = bs.bucket_boundaries(8.0, 2.0)
    mids = np.concatenate([[9.0], (levels[:-1] + levels[1:]) / 2, [0.05]])      # 32 magnitudes, one per bucket
    xs = np.tile(mids, 32).astype(np.float16)
    perm = g.permutation(1024)
    xs = xs[perm]
    for kc in (1, 5, 31):
        m = kc * 32                               # whole buckets only: no overflow
        a = oracle.topk_bucket(xs, m, 8.0, 2.0)
        assert np.array_equal(a, oracle.topk_abs(xs, m))
    assert np.array_equal(oracle.topk_bucket(x, 1024, b0, b15), np.arange(K))
    assert len(oracle.topk_bucket(x, 0, b0, b15)) == 0


def test_calibration_rule():
    g = np.random.default_rng(8)
    X = g.standard_normal((5, 2048)).astype(np.float16)
    k = 40
    b0, b15 = oracle.calibrate_boundaries(X, k)
    kth = [sorted((abs(float(v)) for v in row), reverse=True)[k - 1] for row in X]
    assert float(b15) == max(kth)
    assert float(b0) == max(abs(float(v)) for v in X.ravel())
    assert b0.dtype == np.float32 and b15.dtype == np.float32


def test_recall_against_exact_topk_on_outlier_activations():
    """Section 5.2 reports about 80 % recall against the exact Top-K on real
    activations; the synthetic activations used here must land in the same
    region (recorded, not a parity pin)."""
    import workloads
    K, kc = 4096, 32
    X = np.stack([workloads.x_gauss_outliers(3, 0, "attn_in", 1000 + s, K) for s in range(16)])
    b0, b15 = oracle.calibrate_boundaries(X, kc * 4)
    r = []
    for s in range(20):
        x = workloads.x_gauss_outliers(3, 0, "attn_in", s, K)
        r.append(oracle.recall(oracle.topk_bucket(x, kc, b0, b15), oracle.topk_abs(x, kc * 4)))
    assert 0.6 <= np.mean(r) <= 1.0
    assert oracle.recall(np.array([1, 2, 3]), np.array([2, 3, 4, 5])) == 0.5
