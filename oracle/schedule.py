"""CPU oracle of the offloading-interval rule -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file.  It shares no code with the HIP path and imports nothing from it.

Contents (all exact integer arithmetic; times are nanoseconds):

  offloaded_layers / trigger_layers  placement for an interval N        (Sec. 4.3)
  timeline                           iteration time under that placement (Sec. 4.3, Fig. 7)
  pick_interval                      smallest N that meets the SLO       (Sec. 4.3 last par., 4.4)
  resident_bytes / max_interval      GPU-capacity bound on N             (Sec. 4.5)
  max_tokens                         "max length" a GPU can hold at N    (Sec. 5.6, Fig. 14)
  paper_rule                         the analyzer's closed form          (Sec. 4.4)

Layers are 0-indexed here; the paper counts from 1.

Readings of the paper taken here (each listed in the design notes):
  * interval N: in every group of N consecutive layers the last one is host
    resident; a trailing group shorter than N keeps all its layers on the GPU.
  * the load of an offloaded layer is issued when compute reaches the first layer
    of its group (Sec. 4.3).  For N = 1 that would be the layer itself, yet the
    paper says N = 1 behaves like DeepSpeed, which fetches one layer ahead; so the
    trigger is the previous layer when N = 1.
  * one copy stream, served in issue order; an iteration starts with nothing in
    flight.
  * the analyzer's printed formula divides one layer's compute time by one layer's
    transfer time, which is zero in the paper's own regime (transfer 3.5x / 13.8x
    compute, Sec. 3.2).  It is read with the whole iteration's budget in the
    numerator, and the interval is rounded so that no more than L_offload layers
    are offloaded.  It is reported, never used for the decision.

Parity pins (tests/test_oracle_schedule.py): Fig. 7's worked example, closed forms
for uniform times, a separately written two-queue event simulation, brute force on
tiny cases, monotonicity in the SLO, Table 1's shape.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


# ---------------------------------------------------------------------------
# placement (Sec. 4.3, "Offloading interval")
# ---------------------------------------------------------------------------

def offloaded_layers(L: int, N: int) -> List[int]:
    """Host-resident layers for interval N: the last layer of every full group of N.
    N <= 0 or N > L: nothing is offloaded."""
    if N <= 0 or N > L:
        return []
    return [l for l in range(L) if (l + 1) % N == 0]


PAPER, EAGER, CONTINUOUS = 0, 1, 2     # when the load of an offloaded layer is issued

CONTINUOUS_ITERATIONS = 16              # iterations walked to reach the continuous schedule's steady state


def trigger_layers(L: int, N: int, schedule: int = PAPER) -> List[int]:
    """For each offloaded layer (same order), the layer at whose start its load is issued.

    PAPER: the first layer of the offloaded layer's own group (Sec. 4.3, Fig. 7).
    EAGER: one group earlier -- as early as two staging slots allow: the slot of the k-th
    offloaded layer is free as soon as the (k-2)-th has been computed, so its load is issued at
    the layer after that one (at the start of the iteration for the first two).  This keeps
    the copy stream busy back to back, the regime the analyzer's closed form (Sec. 4.4)
    describes.
    CONTINUOUS: within an iteration the same as EAGER; in addition the loads do not stop at the
    iteration boundary (see timeline_continuous)."""
    back = max(N - 1, 1) if schedule == PAPER else 2 * N - 1
    return [max(0, o - back) for o in offloaded_layers(L, N)]


# ---------------------------------------------------------------------------
# iteration timeline (Fig. 7: compute stream above, copy stream below, sync
# point before each offloaded layer)
# ---------------------------------------------------------------------------

def timeline(tc: Sequence[int], tx: Sequence[int], N: int, schedule: int = PAPER) -> Tuple[int, List[int]]:
    """Iteration time and the stall before each offloaded layer.

    tc[l]: compute time of layer l; tx[l]: host-to-GPU transfer time of layer l's state.
    """
    if schedule == CONTINUOUS:
        times, stalls = timeline_continuous(tc, tx, N, CONTINUOUS_ITERATIONS)
        return max(times[-2:]), stalls
    L = len(tc)
    off = offloaded_layers(L, N)
    trig = trigger_layers(L, N, schedule)
    t = 0                 # compute-stream clock
    copy_free = 0         # time the copy stream finishes what it has been given
    ready = {}            # offloaded layer -> time its state is on the GPU
    stalls = []
    for l in range(L):
        for o, g in zip(off, trig):
            if g == l:
                start = max(copy_free, t)
                copy_free = start + tx[o]
                ready[o] = copy_free
        if l in ready:
            stall = max(0, ready[l] - t)
            stalls.append(stall)
            t += stall
        t += tc[l]
    return t, stalls


def timeline_continuous(tc: Sequence[int], tx: Sequence[int], N: int, iterations: int) -> Tuple[List[int], List[int]]:
    """Back-to-back iterations of the same kind with loads that run on across the iteration
    boundary (the paper is silent on what happens there; its closed form in Sec. 4.4 counts
    how many layer transfers fit into one iteration, which presumes exactly this).

    All loads of all iterations form one sequence g = 0, 1, 2, ...: iteration g // K, the
    (g % K)-th offloaded layer.  Load g goes into staging slot g % 2.  It is issued when the
    layer of load g - m has been computed, m = min(2, K): for K >= 2 that is when its slot
    is given back; for K = 1 the other slot is free all along, but the layer's KV rows of the
    previous iteration must have been written before they are fetched again.  The first m
    loads are issued at time 0.  One copy stream, served in issue order.

    Returns the duration of each iteration and the stalls of the last one.  The first
    iteration starts cold; `timeline` reports the larger of the last two durations."""
    L = len(tc)
    off = offloaded_layers(L, N)
    K = len(off)
    if K == 0:
        return [sum(tc)] * iterations, []
    m = min(2, K)
    computed = {}         # load number -> time its layer finished computing
    ready = {}            # load number -> time its state is on the GPU
    copy_free = 0
    issued = 0            # loads handed to the copy stream so far

    def issue_what_is_due(now: int):
        nonlocal issued, copy_free
        while issued < iterations * K and (issued < m or (issued - m) in computed):
            at = 0 if issued < m else computed[issued - m]
            assert at <= now
            start = max(copy_free, at)
            copy_free = start + tx[off[issued % K]]
            ready[issued] = copy_free
            issued += 1

    t = 0
    times, stalls = [], []
    for it in range(iterations):
        begin = t
        stalls = []
        for l in range(L):
            issue_what_is_due(t)
            if l in off:
                g = it * K + off.index(l)
                stall = max(0, ready[g] - t)
                stalls.append(stall)
                t += stall
                t += tc[l]
                computed[g] = t
            else:
                t += tc[l]
        times.append(t - begin)
    return times, stalls


def hidden_fraction(tx: Sequence[int], N: int, stalls: Sequence[int]) -> float:
    """Share of transfer time that did not delay compute (1.0 when nothing is offloaded)."""
    tot = sum(tx[o] for o in offloaded_layers(len(tx), N))
    return 1.0 if tot == 0 else 1.0 - sum(stalls) / tot


# ---------------------------------------------------------------------------
# GPU-capacity bound (Sec. 4.5: maximum interval from the memory of the GPU)
# ---------------------------------------------------------------------------

def resident_bytes(L: int, N: int, state_bytes: int, slot_bytes: int, fixed_bytes: int) -> int:
    """GPU bytes held for interval N: resident layers' state, two staging slots when
    anything is offloaded, plus what does not depend on N (workspace)."""
    K = len(offloaded_layers(L, N))
    return (L - K) * state_bytes + (2 * slot_bytes if K else 0) + fixed_bytes


STATE, WEIGHTS, KV = 0, 1, 2      # which part of a host-resident layer's state lives on the host


def resident_bytes_of(L: int, N: int, weight_bytes: int, kv_bytes: int, fixed_bytes: int, what: int = STATE) -> int:
    """GPU bytes held for interval N when a host-resident layer keeps on the host its whole state
    (weights and KV slice; Sec. 1 and 2.3 speak of "LLM state"), only its weights, or only its KV
    slice.  The part that stays behind lives on the GPU; a staging slot holds only the part that
    travels."""
    K = len(offloaded_layers(L, N))
    stays = {STATE: 0, WEIGHTS: kv_bytes, KV: weight_bytes}[what]
    travels = weight_bytes + kv_bytes - stays
    return (L - K) * (weight_bytes + kv_bytes) + K * stays + (2 * travels if K else 0) + fixed_bytes


def max_interval(L: int, budget: int, state_bytes: int, slot_bytes: int, fixed_bytes: int) -> int:
    """Largest interval whose footprint fits the budget; L+1 stands for "no offloading"
    (infinite maximum, Sec. 4.5); 0 when not even N = 1 fits.  budget <= 0: no cap."""
    if budget <= 0:
        return L + 1
    best = 0
    for N in range(1, L + 2):
        if resident_bytes(L, N, state_bytes, slot_bytes, fixed_bytes) <= budget:
            best = N
    return best


def max_interval_of(L: int, budget: int, weight_bytes: int, kv_bytes: int, fixed_bytes: int, what: int = STATE) -> int:
    """max_interval for a given choice of what is kept on the host."""
    if budget <= 0:
        return L + 1
    best = 0
    for N in range(1, L + 2):
        if resident_bytes_of(L, N, weight_bytes, kv_bytes, fixed_bytes, what) <= budget:
            best = N
    return best


def max_tokens(L: int, N: int, weight_bytes: int, kv_token_bytes: int, fixed_bytes: int, budget: int,
               what: int = STATE) -> int:
    """Sec. 5.6's "max length" (batch size x (sequence + output length)): the largest number of
    cached tokens for which interval N still fits the budget.  A layer's state is its weights plus
    its KV slice of that many tokens; GPU-resident layers hold one such state, and so does each of
    the two staging slots (when anything is offloaded) -- or only the part of it that travels, when
    host-resident layers keep the other part on the GPU.  Plain search from the definition."""
    def fits(t: int) -> bool:
        return resident_bytes_of(L, N, weight_bytes, t * kv_token_bytes, fixed_bytes, what) <= budget
    if not fits(0):
        return 0
    if kv_token_bytes == 0:
        raise ValueError("unbounded")
    hi = 1
    while fits(hi):
        hi *= 2
    lo = hi // 2                      # fits(lo), not fits(hi)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if fits(mid):
            lo = mid
        else:
            hi = mid
    return lo


def load_bytes(weight_bytes: int, kv_prefix_bytes: int, what: int = STATE) -> int:
    """Bytes one host-resident layer's load moves host-to-GPU: the part of its state that lives on
    the host (kv_prefix_bytes: its cached K/V so far; 0 in a prefill from empty caches)."""
    return {STATE: weight_bytes + kv_prefix_bytes, WEIGHTS: weight_bytes, KV: kv_prefix_bytes}[what]


# ---------------------------------------------------------------------------
# picker: the optimal interval is the smallest one that meets the SLO (Sec. 4.3,
# 4.4); the request is rejected when minimum > maximum (Sec. 4.5, Fig. 8)
# ---------------------------------------------------------------------------

def min_interval(tc: Sequence[int], tx: Sequence[int], slo: int, schedule: int = PAPER) -> Optional[int]:
    """Smallest N in 1..L with iteration time <= slo; L+1 if only the un-offloaded
    iteration meets it; None if even that does not."""
    L = len(tc)
    for N in range(1, L + 1):
        if timeline(tc, tx, N, schedule)[0] <= slo:
            return N
    return L + 1 if sum(tc) <= slo else None


def pick_interval(tc: Sequence[int], tx: Sequence[int], slo: int, n_max: int, schedule: int = PAPER) -> Optional[int]:
    """The interval to run with, or None when the SLO cannot be met within capacity."""
    n_min = min_interval(tc, tx, slo, schedule)
    if n_min is None or n_min > n_max:
        return None
    return n_min


def refine_interval(tc: Sequence[int], tx: Sequence[int], N: int, schedule: int = PAPER) -> int:
    """Among the intervals that keep as many layers on the host as N does, the one whose iteration is shortest
    (the smallest such interval on a tie; N itself is a candidate).

    The paper's objective is host memory: a smaller interval is better because it offloads more layers (Sec. 4.3),
    and the optimal interval is the smallest that meets the SLO (Sec. 4.4).  Where L is not a multiple of N several
    intervals offload the same floor(L / N) layers -- the same host memory, the same GPU footprint -- and the paper
    does not choose between them; this does, by iteration time.  The result offloads what N offloads and is never
    slower, so it meets every SLO and capacity bound that N meets.  N = L + 1 (nothing offloaded) stays."""
    L = len(tc)
    if N > L:
        return N
    K = L // N
    best_n, best_t = N, timeline(tc, tx, N, schedule)[0]
    for cand in range(N + 1, L + 1):
        if L // cand != K:
            break
        t = timeline(tc, tx, cand, schedule)[0]
        if t < best_t:
            best_n, best_t = cand, t
    return best_n


# ---------------------------------------------------------------------------
# the analyzer's closed form (Sec. 4.4, "Design"), reported beside the pick
# ---------------------------------------------------------------------------

def paper_rule(L: int, t_compute: int, t_trans: int, slo: int) -> int:
    """L_offload = floor(slo / t_trans) layer transfers fit a saturated copy stream
    within the SLO (slo = (1 + delta) * L * t_compute); the interval is the smallest N
    that offloads no more than that: floor(L / (L_offload + 1)) + 1."""
    if t_trans <= 0:
        return 1
    l_off = slo // t_trans
    return L // (l_off + 1) + 1


def paper_rule_as_printed(L: int, t_compute: int, t_trans: int, delta_num: int, delta_den: int):
    """The formula exactly as printed: L_offload = floor(t_compute (1+delta) / t_trans),
    interval = floor(L / L_offload).  None where it divides by zero."""
    l_off = (t_compute * (delta_den + delta_num)) // (t_trans * delta_den)
    return None if l_off == 0 else L // l_off
