"""CPU oracle of the per-bus bandwidth coordinator -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file.  It shares no code with the HIP path and imports nothing from it.

Sec. 4.5 / Fig. 8: GPU instances that share a host link each have a minimum interval
(below it the request's SLO is violated; from the performance record) and a maximum
interval (above it the model no longer fits the GPU; "infinite" if it fits entirely).
The interval also fixes the link bandwidth an instance consumes.  The coordinator picks,
for every instance, an interval within [min, max] such that the consumed bandwidths sum
to less than the link's, maximising the total host memory in use.

Readings of the paper taken here (each listed in the design notes):
  * layers offloaded at interval N: floor(L / N) (the figure divides `layers / intv` as
    reals; the placement of Sec. 4.3 offloads whole layers), none for N = L + 1, which
    stands for "no offloading" and is a legal choice only when max is L + 1 (infinite).
  * bandwidth of an instance: offloaded layers x bytes per layer, once per iteration,
    i.e. K(N) * mem_per_layer / iter_time, in integer bytes per second (rounded down).
  * valid: the sum is STRICTLY below the link bandwidth, as the figure prints it.
  * the figure's first check (request min > instance max: reject) applies to every
    instance; if no combination is valid the adjustment fails as well.
  * ties between combinations of equal host memory (the paper is silent): the one that
    consumes less bandwidth, then the lexicographically smallest tuple of intervals.
  * the figure enumerates two instances and says more are analogous: any number here.

This is the plain definition: every combination of intervals is enumerated.
Parity pins (tests/test_oracle_coordinator.py): hand-worked two-instance cases, the idle
neighbour special case (the request is served with its minimum interval), bounds.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple


@dataclass(frozen=True)
class Instance:
    n_layers: int
    mem_per_layer: int      # bytes moved per offloaded layer per iteration
    iter_ns: int            # iteration time the rate is computed with (Fig. 8: iter_time)
    n_min: int              # smallest interval that meets the SLO
    n_max: int              # largest interval the GPU's capacity allows; n_layers + 1: infinite


def offloaded(inst: Instance, N: int) -> int:
    return inst.n_layers // N if 1 <= N <= inst.n_layers else 0


def host_bytes(inst: Instance, N: int) -> int:
    return offloaded(inst, N) * inst.mem_per_layer


def rate(inst: Instance, N: int) -> int:
    """Link bandwidth consumed at interval N, bytes per second (Fig. 8, is_valid)."""
    return host_bytes(inst, N) * 1_000_000_000 // inst.iter_ns


def adjust(instances: Sequence[Instance], bandwidth: int) -> Optional[Tuple[Tuple[int, ...], int, int]]:
    """(intervals, total host bytes, total bytes/s) of the best valid combination, or None."""
    ranges: List[range] = []
    for g in instances:
        hi = min(g.n_max, g.n_layers + 1)
        if g.n_min < 1 or g.n_min > hi:
            return None                                   # SLO cannot be met within capacity: reject
        ranges.append(range(g.n_min, hi + 1))
    best = None
    for combo in itertools.product(*ranges):
        r = sum(rate(g, n) for g, n in zip(instances, combo))
        if not r < bandwidth:
            continue
        m = sum(host_bytes(g, n) for g, n in zip(instances, combo))
        key = (-m, r, combo)
        if best is None or key < best[0]:
            best = (key, combo, m, r)
    return None if best is None else (tuple(best[1]), best[2], best[3])
