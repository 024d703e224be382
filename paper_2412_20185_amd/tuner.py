"""The DecDEC parameter tuner (Section 4.4) and the small analytical models of
the paper, as host-side logic.

The tuner picks, for a target slowdown over the uncompensated model, how many
fetch workgroups each type of linear layer gets (n_tb) and how many channels
per 1024 it compensates (k_chunk).  It only needs a function that returns the
time of all linear layers for a given configuration; on the GPU that function
replays a captured layer (see `python -m paper_2412_20185_amd.microbench tune`),
in the tests it is a synthetic cost model.

Phase 1 replaces the per-type n_tb by one cap n_tb^max (each type takes its
largest candidate not above the cap) and, for every cap up to half the number
of compute units, counts how many uniform +1 steps of k_chunk on all types stay
within the budget; the cap with the most steps wins.  If no cap admits a single
step, the type with the smallest weight matrix is frozen at k_chunk = 0 and the
search repeats.  Phase 2 starts from that uniform k_chunk and raises the types
one by one, cheapest increase first, until no type can be raised.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Dict, List, Sequence, Tuple


def ntb_candidates(d_in: int, d_out: int) -> List[int]:
    """Thread-block counts worth trying for one layer type (Section 4.4,
    "Technical Details"): A = {1 .. d_in/1024} (one chunk is the smallest unit
    of the selection) united with B = {n <= s : ceil(s / ceil(s / n)) = n},
    s = d_out/256 segments of 256 4-bit residuals (only the smallest n for every
    distinct number of segments per block)."""
    A = set(range(1, d_in // 1024 + 1))
    s = d_out // 256
    Bset = {n for n in range(1, s + 1) if math.ceil(s / math.ceil(s / n)) == n}
    return sorted(A | Bset)


def kchunk_max_for_shared_memory(bytes_per_block: int) -> int:
    """Largest k_chunk of the paper's kernel: 128 B of bucket counters,
    128 * k_chunk B of per-bucket index lists and 2 * 1024 B of activations must
    fit in the block's shared memory (Section 4.4)."""
    return (bytes_per_block - 128 - 2 * 1024) // 128


def knee_kchunk(r_bw: float, weight_bits: int, residual_bits: int = 4) -> float:
    """k_chunk up to which the compensation hides behind the base GEMV when both
    run at full bandwidth (Section 5.1): 1024 * (1 / R_bw) * (b / r), R_bw =
    memory bandwidth / host-link bandwidth; the paper states it for r = 4."""
    return 1024.0 / r_bw * weight_bits / residual_bits


@dataclass(frozen=True)
class LayerType:
    name: str
    d_in: int
    d_out: int
    candidates: Tuple[int, ...] = ()

    def ntb_options(self) -> List[int]:
        return list(self.candidates) if self.candidates else ntb_candidates(self.d_in, self.d_out)

    def weight_elems(self) -> int:
        return self.d_in * self.d_out


Config = Dict[str, Tuple[int, int]]  # type name -> (n_tb, k_chunk)
Measure = Callable[[Config], float]


def ntb_for_cap(types: Sequence[LayerType], cap: int) -> Dict[str, int]:
    """Each type's largest candidate not above the cap (its smallest if none is)."""
    out = {}
    for t in types:
        opts = t.ntb_options()
        below = [n for n in opts if n <= cap]
        out[t.name] = max(below) if below else min(opts)
    return out


@dataclass
class TunerResult:
    ntb_max: int
    ntb: Dict[str, int]
    k_chunk: Dict[str, int]
    baseline: float
    time: float
    coarse_steps: int
    frozen: List[str]

    @property
    def slowdown(self) -> float:
        return self.time / self.baseline - 1.0


def tune(types: Sequence[LayerType], measure: Measure, target_slowdown: float, ntb_max_limit: int,
         k_chunk_limit: int = 1024) -> TunerResult:
    """Runs both phases.  `measure(config)` returns the time of all linear
    layers with the given (n_tb, k_chunk) per type; k_chunk = 0 everywhere is the
    baseline.  ntb_max_limit: the paper tests caps up to half the SM count."""
    names = [t.name for t in types]
    base_cfg = {n: (1, 0) for n in names}
    baseline = measure(base_cfg)
    budget = baseline * (1.0 + target_slowdown)

    frozen: List[str] = []
    order_small_first = [t.name for t in sorted(types, key=lambda t: t.weight_elems())]
    while True:
        active = [n for n in names if n not in frozen]
        best = (-1, 1, ntb_for_cap(types, 1))
        if active:
            for cap in range(1, max(1, ntb_max_limit) + 1):
                ntb = ntb_for_cap(types, cap)
                steps = 0
                while steps < k_chunk_limit:
                    cfg = {n: (ntb[n], steps + 1 if n in active else 0) for n in names}
                    if measure(cfg) > budget:
                        break
                    steps += 1
                if steps > best[0]:
                    best = (steps, cap, ntb)
        if best[0] > 0 or not active:
            break
        frozen.append(next(n for n in order_small_first if n not in frozen))   # smallest matrix first
    steps, cap, ntb = best
    steps = max(steps, 0)
    k = {n: (steps if n not in frozen else 0) for n in names}

    # Phase 2: raise single types, cheapest increase first, until none fits.
    final = set(frozen)
    current = measure({n: (ntb[n], k[n]) for n in names})
    while len(final) < len(names):
        trial = []
        for n in names:
            if n in final:
                continue
            if k[n] >= k_chunk_limit:
                final.add(n)
                continue
            cfg = {m: (ntb[m], k[m] + (1 if m == n else 0)) for m in names}
            trial.append((measure(cfg) - current, n))
        progressed = False
        for _, n in sorted(trial):
            cfg = {m: (ntb[m], k[m] + (1 if m == n else 0)) for m in names}
            t = measure(cfg)
            if t <= budget:
                k[n] += 1
                current = t
                progressed = True
            else:
                final.add(n)
        if not progressed:
            break
    return TunerResult(ntb_max=cap, ntb=ntb, k_chunk=k, baseline=baseline, time=current, coarse_steps=steps,
                       frozen=frozen)
