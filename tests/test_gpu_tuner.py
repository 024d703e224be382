"""The parameter tuner of Section 4.4 driven by real measurements on the GPU: one Llama-3-8B-shaped
layer (3-bit weights, fp16 host residuals), measure() = wall time of the layer's four calls replayed
as a captured graph, target slowdowns of 10 % and 30 % over the uncompensated layer."""
import pytest

from paper_2412_20185_amd import tuner as T
from paper_2412_20185_amd.microbench import LayerHarness

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(600)
@pytest.mark.parametrize("target", [0.10, 0.30])
def test_tuned_configuration_meets_the_target_and_is_maximal(target):
    h = LayerHarness("8b", reps=30)
    try:
        r = T.tune(h.types, h.measure, target, ntb_max_limit=64, k_chunk_limit=128)
        names = [t.name for t in h.types]
        budget = r.baseline * (1.0 + target)
        cfg = {n: (r.ntb[n], r.k_chunk[n]) for n in names}
        print(f"tuned: split {r.ntb}, k_chunk {r.k_chunk}, baseline {r.baseline:.1f} us, tuned {r.time:.1f} us "
              f"(+{100 * r.slowdown:.1f} %), frozen {r.frozen}, {len(h.cache)} configurations measured")
        # what the tuner returns is what it measured, and that is inside the budget
        assert r.time == h.measure(cfg) and r.time <= budget
        assert all(r.ntb[n] in (1, 2, 4, 8, 16, 32, 64) and 0 <= r.k_chunk[n] <= 128 for n in names)
        # maximal: one more channel per 1024 on any type the tuner was still raising breaks the budget
        # (the measurements the tuner itself took; a frozen type stays at 0 by the algorithm's rule)
        for n in names:
            if n in r.frozen:
                assert r.k_chunk[n] == 0
                continue
            more = {m: (r.ntb[m], r.k_chunk[m] + (1 if m == n else 0)) for m in names}
            assert h.measure(more) > budget, (n, h.measure(more), budget)
        # measured afresh through the library, the tuned layer stays within the target (3 points of
        # slack for run-to-run timing noise) and the uncompensated layer has not moved
        base_again = h.time_once({n: (1, 0) for n in names})
        tuned_again = h.time_once(cfg)
        assert abs(base_again / r.baseline - 1.0) < 0.05, (base_again, r.baseline)
        assert tuned_again / base_again - 1.0 <= target + 0.03, (tuned_again, base_again)
        # the machine's knee (Section 5.1) is below one channel per 1024 for fp16 residuals, so budgets like
        # these buy only a few channels (none at all where one channel already costs more than the budget)
        assert max(r.k_chunk.values()) <= 8
        if target >= 0.30:
            assert max(r.k_chunk.values()) >= 1
    finally:
        h.close()
