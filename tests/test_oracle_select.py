"""Pins for oracle.topk_abs (Section 4.1 step 1; exact Top-K of Section 5.2).

The pin is a brute force that never sorts: it repeatedly scans for the largest
remaining |x| as a Python float, taking the first (lowest-index) maximum.
Planted mistakes (tie to the higher index, signed instead of absolute value,
k off by one, unsorted output) must each fail the same check.
"""
import numpy as np
import pytest

from oracle import topk_abs, magnitude_keys


def brute_topk(x16, k):
    vals = [abs(float(v)) for v in x16]
    taken = [False] * len(vals)
    out = []
    for _ in range(k):
        best, bi = -1.0, -1
        for i, v in enumerate(vals):
            if not taken[i] and v > best:      # strict: first maximum wins
                best, bi = v, i
        taken[bi] = True
        out.append(bi)
    return sorted(out)


def cases():
    g = np.random.default_rng(7)
    yield "gauss", g.standard_normal(97).astype(np.float16), [0, 1, 5, 96, 97]
    yield "all_equal", np.full(33, 1.5, np.float16), [0, 1, 7, 33]
    dup = g.integers(-3, 4, size=200).astype(np.float16)       # 7 distinct values, many ties
    yield "many_duplicates", dup, [0, 1, 10, 50, 120, 199, 200]
    pm = np.array([0.0, -0.0, 1.0, -1.0, 0.0, -0.0, -1.0, 1.0], np.float16)
    yield "signed_zero_and_pairs", pm, list(range(9))
    sub = np.array([6e-8, -6e-8, 1.2e-7, 0, 6.1e-5, -6.0e-5, 65504, -65504], np.float16)
    yield "subnormal_and_max", sub, list(range(9))
    yield "single", np.array([-2.0], np.float16), [0, 1]
    yield "empty", np.zeros(0, np.float16), [0]


@pytest.mark.parametrize("name,x,ks", list(cases()), ids=[c[0] for c in cases()])
def test_topk_matches_brute_force(name, x, ks):
    for k in ks:
        got = topk_abs(x, k)
        assert got.dtype == np.int32
        assert got.tolist() == brute_topk(x, k), (name, k)


def check_selector(sel):
    """True when `sel` agrees with brute force on the adversarial cases."""
    for _, x, ks in cases():
        for k in ks:
            try:
                got = list(np.asarray(sel(x, k)).tolist())
            except Exception:
                return False
            if got != brute_topk(x, k):
                return False
    return True


def test_planted_mistakes_are_caught():
    assert check_selector(topk_abs)

    def tie_high(x, k):
        key = magnitude_keys(x)
        order = np.argsort(-key[::-1], kind="stable")
        return np.sort(len(key) - 1 - order[:k])

    def signed(x, k):
        order = np.argsort(-x.astype(np.float64), kind="stable")
        return np.sort(order[:k])

    def off_by_one(x, k):
        return topk_abs(x, min(k + 1, len(x)))

    def unsorted(x, k):
        key = magnitude_keys(x)
        return np.argsort(-key, kind="stable")[:k]

    for bad in (tie_high, signed, off_by_one, unsorted):
        assert not check_selector(bad), bad.__name__


def test_keys_order_like_absolute_value_for_every_fp16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bits.view(np.float16)
    ok = ~np.isnan(x)
    key = magnitude_keys(x)[ok].astype(np.int64)
    a = np.abs(x[ok].astype(np.float64))
    order = np.argsort(key, kind="stable")
    ks, as_ = key[order], a[order]
    assert np.all(as_[1:] >= as_[:-1])                        # monotone
    # strictly: equal keys <=> equal magnitudes
    assert np.array_equal(ks[1:] == ks[:-1], as_[1:] == as_[:-1])
    # NaN patterns rank above infinity
    assert magnitude_keys(x[~ok]).min() > magnitude_keys(np.array([np.inf], np.float16))[0]


def test_threshold_invariants_random():
    g = np.random.default_rng(11)
    for K, k in [(1024, 32), (4096, 81), (14336, 286), (4096, 4095)]:
        x = (g.standard_t(3, size=K)).astype(np.float16)
        sc = topk_abs(x, k)
        a = np.abs(x.astype(np.float64))
        mask = np.zeros(K, bool)
        mask[sc] = True
        assert len(sc) == k and np.all(np.diff(sc) > 0)
        thr = a[mask].min()
        assert thr >= a[~mask].max()
        # every excluded element equal to the threshold has a higher index than every included one equal to it
        inc_eq = np.nonzero(mask & (a == thr))[0]
        exc_eq = np.nonzero(~mask & (a == thr))[0]
        if len(exc_eq):
            assert inc_eq.max() < exc_eq.min()


def test_scaling_by_two_keeps_selection():
    g = np.random.default_rng(5)
    x = g.standard_normal(2048).astype(np.float16)
    assert np.array_equal(topk_abs(x, 100), topk_abs((x * np.float16(2)).astype(np.float16), 100))
