"""The paper's tuner and analytical models (Sections 4.4, 5.1), pinned to the
numbers the paper prints and checked on a synthetic cost model."""
import math

import pytest

from paper_2412_20185_amd import tuner as T


def test_candidate_set_printed_for_llama3_8b_qkv():
    """Section 4.4: for Llama-3-8B the fused q/k/v layer (4096 x 6144) has the 9
    candidates 1, 2, 3, 4, 5, 6, 8, 12, 24."""
    assert T.ntb_candidates(4096, 6144) == [1, 2, 3, 4, 5, 6, 8, 12, 24]


def test_ntb_for_cap_against_the_figure_11_example():
    """Figure 11(b): n_tb^max = 24 gives (n_qkv, n_o, n_gu, n_d) = (24, 16, 23, 14).
    The printed rule ("largest candidate below n_tb^max") reproduces the first
    three; for the down projection (14336 x 4096) it gives 16, because 16 = s is
    in set B, while the figure prints 14 = d_in/1024, the largest member of set A:
    an inconsistency inside the paper, recorded here."""
    types = [T.LayerType("qkv", 4096, 6144), T.LayerType("o", 4096, 4096),
             T.LayerType("gu", 4096, 28672), T.LayerType("d", 14336, 4096)]
    got = T.ntb_for_cap(types, 24)
    assert (got["qkv"], got["o"], got["gu"]) == (24, 16, 23)
    assert got["d"] == 16
    assert 14 in T.ntb_candidates(14336, 4096) and 15 not in T.ntb_candidates(14336, 4096)


def test_shared_memory_bound_and_knee_model():
    """Section 4.4: 48 KB of shared memory allow k_chunk up to 367.  Section 5.1:
    R_bw = 12 (RTX 4050M) and 3-bit weights put the knee at k_chunk = 64."""
    assert T.kchunk_max_for_shared_memory(49152) == 367
    assert 128 + 128 * 367 + 2 * 1024 <= 49152 < 128 + 128 * 368 + 2 * 1024
    assert T.knee_kchunk(12, 3) == pytest.approx(64.0)
    assert T.knee_kchunk(32, 3) == pytest.approx(24.0)          # RTX 4090
    assert T.knee_kchunk(12, 4) == pytest.approx(1024 / 12)     # "4/4 = 1 for 4-bit quantization"


def cost_model(link_rows_per_us=2.0):
    """Per type: base time b; compensation needs k_chunk * d_in/1024 rows of d_out values over a link that
    n_tb blocks fill up to min(1, n_tb/8); the part of it beyond the base time shows; each block slows the
    base GEMV by 0.2 %."""
    shapes = {"qkv": (4096, 6144, 10.0), "o": (4096, 4096, 7.0), "gu": (4096, 28672, 40.0), "d": (14336, 4096, 20.0)}

    def measure(cfg):
        total = 0.0
        for name, (n_tb, kc) in cfg.items():
            d_in, d_out, base = shapes[name]
            gemv = base * (1 + 0.002 * n_tb * (kc > 0))
            rows = kc * d_in // 1024
            dec = rows * d_out / 4096 / (link_rows_per_us * min(1.0, n_tb / 8)) + (1.0 if kc else 0.0)
            total += max(gemv, dec)
        return total
    types = [T.LayerType(n, s[0], s[1]) for n, s in shapes.items()]
    return types, measure


@pytest.mark.parametrize("target", [0.025, 0.05, 0.1, 0.2])
def test_tuner_meets_the_target_and_is_maximal(target):
    types, measure = cost_model()
    r = T.tune(types, measure, target, ntb_max_limit=28)
    cfg = {t.name: (r.ntb[t.name], r.k_chunk[t.name]) for t in types}
    assert measure(cfg) <= r.baseline * (1 + target) + 1e-9
    assert r.slowdown <= target + 1e-12
    assert all(v >= 0 for v in r.k_chunk.values()) and max(r.k_chunk.values()) > 0
    for t in types:                                  # no single type can take one more channel per chunk
        bumped = dict(cfg)
        bumped[t.name] = (cfg[t.name][0], cfg[t.name][1] + 1)
        assert measure(bumped) > r.baseline * (1 + target)
    assert all(r.ntb[t.name] in t.ntb_options() and r.ntb[t.name] <= max(r.ntb_max, min(t.ntb_options())) for t in types)
    assert min(r.k_chunk.values()) >= r.coarse_steps or r.frozen      # phase 2 only raises


def test_tuner_is_monotone_in_the_target_and_freezes_small_layers_when_nothing_fits():
    types, measure = cost_model()
    ks = [sum(T.tune(types, measure, t, 28).k_chunk.values()) for t in (0.025, 0.05, 0.1, 0.2)]
    assert ks == sorted(ks) and ks[-1] > ks[0]
    # a link so slow that a uniform step never fits: the smallest layers are frozen at 0 one after the other
    types, slow = cost_model(link_rows_per_us=0.02)
    r = T.tune(types, slow, 0.01, 28)
    assert r.slowdown <= 0.01 + 1e-12
    assert r.frozen[:1] == ["o"]                      # 4096 x 4096 is the smallest weight matrix
    assert all(r.k_chunk[n] == 0 for n in r.frozen)
