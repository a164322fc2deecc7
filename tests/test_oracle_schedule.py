"""Pins for oracle/schedule.py: the paper's worked example (Fig. 7), closed forms for
uniform layer times, a separately written two-queue event simulation, hand-worked
numbers, brute force and the invariants the method promises."""
import itertools
import os
import random

import pytest

from oracle import schedule as osch


def _read_kv(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = [int(t) for t in v]
    return out


def test_fig7_worked_example(golden_dir):
    g = _read_kv(os.path.join(golden_dir, "fig7_schedule.txt"))
    L, N = g["layers"][0], g["interval"][0]
    off = osch.offloaded_layers(L, N)
    assert [o + 1 for o in off] == g["offloaded"]
    assert [t + 1 for t in osch.trigger_layers(L, N)] == g["prefetch_issued_before"]
    assert sorted(set(range(1, L + 1)) - {o + 1 for o in off}) == g["gpu_resident"]
    assert [o + 1 for o in off] == g["sync_before"]


def test_config1_placement(golden_dir):
    g = _read_kv(os.path.join(golden_dir, "config1_placement.txt"))
    assert osch.offloaded_layers(g["layers"][0], g["interval"][0]) == g["offloaded_zero_indexed"]


def test_placement_special_cases():
    assert osch.offloaded_layers(6, 1) == [0, 1, 2, 3, 4, 5]       # every layer on the host
    assert osch.trigger_layers(6, 1) == [0, 0, 1, 2, 3, 4]          # fetched one layer ahead
    assert osch.offloaded_layers(6, 7) == [] and osch.offloaded_layers(6, 0) == []
    assert osch.offloaded_layers(10, 4) == [3, 7]                   # trailing 2 layers stay on the GPU
    assert osch.offloaded_layers(10, 10) == [9]
    for L in range(1, 40):
        for N in range(1, L + 3):
            off = osch.offloaded_layers(L, N)
            assert len(off) == (L // N if N <= L else 0)
            for o, g in zip(off, osch.trigger_layers(L, N)):
                assert g == (o - (N - 1) if N > 1 else max(0, o - 1))


def test_timeline_hand_worked():
    # L=4, N=2: layers 1 and 3 offloaded, loads issued at layers 0 and 2.
    # tc = 10 each, tx = 25 each.
    # t=0: load(1) runs 0..25.  layer0 0..10.  layer1 waits until 25 (stall 15), runs 25..35.
    # layer2 starts 35: load(3) runs 35..60; layer2 35..45; layer3 waits to 60 (stall 15), 60..70.
    T, stalls = osch.timeline([10] * 4, [25] * 4, 2)
    assert (T, stalls) == (70, [15, 15])
    # fully hidden when tx <= tc
    assert osch.timeline([10] * 4, [9] * 4, 2) == (40, [0, 0])
    # N=1, L=3, tc=10, tx=25: loads of 0 and 1 issued at layer 0 (0..25, 25..50); load of 2 at
    # layer 1.  layer0 25..35; layer1 starts 35 -> load(2) 50..75; waits to 50, runs 50..60;
    # layer2 waits to 75, runs 75..85.
    assert osch.timeline([10] * 3, [25] * 3, 1) == (85, [25, 15, 15])
    # non-uniform: only the offloaded layers' tx matter
    T, stalls = osch.timeline([5, 7, 11, 13], [1000, 20, 1000, 3], 2)
    assert (T, stalls) == (5 + 15 + 7 + 11 + 13, [15, 0])
    assert osch.hidden_fraction([1000, 20, 1000, 3], 2, stalls) == pytest.approx(1 - 15 / 23)


def test_timeline_degenerate():
    tc = [3, 1, 4, 1, 5, 9, 2, 6]
    assert osch.timeline(tc, [100] * 8, 9)[0] == sum(tc)            # N > L: nothing offloaded
    assert osch.timeline(tc, [100] * 8, 0)[0] == sum(tc)
    for N in range(1, 9):
        assert osch.timeline(tc, [0] * 8, N)[0] == sum(tc)          # free transfers never stall


def test_timeline_closed_forms_uniform():
    rnd = random.Random(1)
    for _ in range(3000):
        L, c, x = rnd.randint(1, 48), rnd.randint(1, 1000), rnd.randint(0, 20000)
        N = rnd.randint(1, L + 1)
        T, stalls = osch.timeline([c] * L, [x] * L, N)
        K = L // N if N <= L else 0
        if N >= 2:
            want = L * c + K * max(0, x - (N - 1) * c)
        else:
            want = x + (L - 1) * max(c, x) + c
        assert T == want, (L, c, x, N)
        if N >= 2 and K and x:
            assert osch.hidden_fraction([x] * L, N, stalls) == pytest.approx(min(1.0, (N - 1) * c / x))


def _two_queue_simulation(tc, tx, N):
    """Independent formulation: build the list of operations each stream is given, with
    explicit cross-stream dependencies, then resolve start/end times by relaxation."""
    L = len(tc)
    off = [l for l in range(L) if N >= 1 and N <= L and (l + 1) % N == 0]
    trig = {o: max(0, o - max(N - 1, 1)) for o in off}
    compute = [("layer", l) for l in range(L)]
    copy = [("load", o) for o in sorted(off, key=lambda o: (trig[o], o))]
    end = {}
    start = {}
    changed = True
    while changed:
        changed = False
        for queue in (compute, copy):
            prev_end = 0
            for op in queue:
                deps = [prev_end]
                kind, l = op
                if kind == "layer" and l in off:
                    deps.append(end.get(("load", l)))
                if kind == "load":
                    g = trig[l]
                    deps.append(start.get(("layer", g)) if g > 0 else 0)
                    if g > 0:
                        # issued when compute *reaches* layer g = when layer g-1 ends
                        deps[-1] = end.get(("layer", g - 1))
                if any(d is None for d in deps):
                    break
                s = max(deps)
                e = s + (tc[l] if kind == "layer" else tx[l])
                if start.get(op) != s or end.get(op) != e:
                    start[op], end[op] = s, e
                    changed = True
                prev_end = e
    return end[("layer", L - 1)]


def test_timeline_equals_independent_event_simulation():
    rnd = random.Random(2)
    for _ in range(1500):
        L = rnd.randint(1, 20)
        tc = [rnd.randint(1, 100) for _ in range(L)]
        tx = [rnd.randint(0, 400) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        assert osch.timeline(tc, tx, N)[0] == _two_queue_simulation(tc, tx, N), (tc, tx, N)


def _slot_simulation(tc, tx, N):
    """The eager schedule from its own definition, without trigger layers: two staging slots; the
    k-th offloaded layer uses slot k % 2; its load starts as soon as the copy stream is free and the
    slot is (i.e. the layer that last used it has been computed); loads are served in layer order."""
    L = len(tc)
    off = [l for l in range(L) if 1 <= N <= L and (l + 1) % N == 0]
    load_end = {}
    layer_end = {}
    t = 0
    copy_free = 0
    k_next = 0                      # next load to hand to the copy stream

    def issue_ready_loads(now):
        nonlocal k_next, copy_free
        while k_next < len(off):
            user = off[k_next - 2] if k_next >= 2 else None       # previous user of this slot
            if user is not None and user not in layer_end:
                break
            slot_free = 0 if user is None else layer_end[user]
            if slot_free > now:
                break
            start = max(copy_free, slot_free)
            copy_free = start + tx[off[k_next]]
            load_end[off[k_next]] = copy_free
            k_next += 1

    issue_ready_loads(0)
    for l in range(L):
        if l in off:
            t = max(t, load_end[l])
        t += tc[l]
        layer_end[l] = t
        issue_ready_loads(t)
    return t


def test_eager_schedule_hand_worked_and_independent_simulation():
    # L = 4, N = 2, compute 10 per layer, transfer 25: layers 1 and 3 are on the host.
    # Paper's schedule: load(1) 0-25; layer 0 0-10; stall to 25; layer 1 25-35; load(3) issued at 35, 35-60;
    #   layer 2 35-45; stall to 60; layer 3 60-70.
    # Eager: both slots are free at the start: load(1) 0-25, load(3) 25-50; layer 1 25-35; layer 2 35-45;
    #   stall to 50; layer 3 50-60.
    tc, tx = [10] * 4, [25] * 4
    assert osch.timeline(tc, tx, 2) == (70, [15, 15])
    assert osch.timeline(tc, tx, 2, osch.EAGER) == (60, [15, 5])
    assert osch.trigger_layers(8, 2, osch.EAGER) == [0, 0, 2, 4] and osch.trigger_layers(8, 2) == [0, 2, 4, 6]
    assert osch.trigger_layers(6, 1, osch.EAGER) == osch.trigger_layers(6, 1)         # N = 1: already one layer ahead
    rnd = random.Random(21)
    for _ in range(3000):
        L = rnd.randint(1, 24)
        tc = [rnd.randint(1, 100) for _ in range(L)]
        tx = [rnd.randint(0, 500) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        eager = osch.timeline(tc, tx, N, osch.EAGER)[0]
        assert eager == _slot_simulation(tc, tx, N), (tc, tx, N)
        paper = osch.timeline(tc, tx, N)[0]
        assert eager <= paper                                   # issuing earlier never hurts
        if L // N <= 1 or N == 1 or N > L:
            assert eager == paper                               # nothing to issue earlier
    # saturated copy stream, uniform times, N | L, x >= N c: the loads run back to back from t = 0 and
    # the last layer computes after the last load: T = K x + c  (the regime of the analyzer's closed form)
    for L, N, c, x in [(8, 2, 10, 25), (12, 3, 7, 40), (32, 4, 5, 21), (6, 2, 3, 6)]:
        assert osch.timeline([c] * L, [x] * L, N, osch.EAGER)[0] == (L // N) * x + c



def _dependency_graph_times(tc, tx, N, iterations):
    """The continuous schedule as a dependency graph, solved by longest paths: compute task (i, l)
    follows the previous compute task and, if layer l is on the host, its load; load g follows load
    g - 1 (one copy stream) and the compute task of load g - min(2, K) (staging slot / KV rows)."""
    L = len(tc)
    off = [l for l in range(L) if 1 <= N <= L and (l + 1) % N == 0]
    K = len(off)
    m = min(2, K)
    load_done, layer_done = {}, {}

    def load(g):
        if g not in load_done:
            after = [0]
            if g >= 1:
                after.append(load(g - 1))
            if g >= m:
                after.append(layer(*divmod(g - m, K)))
            load_done[g] = max(after) + tx[off[g % K]]
        return load_done[g]

    def layer(i, k_or_l, by_layer=False):
        l = k_or_l if by_layer else off[k_or_l]
        if (i, l) not in layer_done:
            after = [0]
            if l > 0:
                after.append(layer(i, l - 1, True))
            elif i > 0:
                after.append(layer(i - 1, L - 1, True))
            if l in off:
                after.append(load(i * K + off.index(l)))
            layer_done[(i, l)] = max(after) + tc[l]
        return layer_done[(i, l)]

    import sys
    sys.setrecursionlimit(100000)
    ends = [0]
    for i in range(iterations):
        for l in range(L):
            layer(i, l, True)                 # in order, so the recursion stays shallow
        ends.append(layer_done[(i, L - 1)])
    return [b - a for a, b in zip(ends, ends[1:])]


def test_continuous_schedule_hand_worked_closed_forms_and_dependency_graph():
    # L = 4, N = 2, compute 10, transfer 25 (layers 1 and 3 on the host), loads numbered across iterations:
    # load0 0-25, load1 25-50; iteration 0: layer0 0-10, layer1 25-35 (-> load2 50-75), layer2 35-45,
    #   layer3 50-60 (-> load3 75-100): 60, as the eager schedule from a cold start.
    # iteration 1: layer0 60-70, layer1 75-85 (-> load4 100-125), layer2 85-95, layer3 100-110 (-> load5 125-150): 50
    # iteration 2: layer0 110-120, layer1 125-135, layer2 135-145, layer3 150-160: 50 = 2 transfers.
    tc, tx = [10] * 4, [25] * 4
    times, stalls = osch.timeline_continuous(tc, tx, 2, 3)
    assert times == [60, 50, 50] and stalls == [5, 5]
    assert osch.timeline(tc, tx, 2, osch.CONTINUOUS) == (50, [5, 5])
    assert osch.trigger_layers(8, 2, osch.CONTINUOUS) == osch.trigger_layers(8, 2, osch.EAGER)
    # one offloaded layer (K = 1): its next load starts when it has been computed, so an iteration is
    # the longer of the compute chain and one transfer plus that layer: max(L c, x + c)
    assert osch.timeline([10] * 6, [100] * 6, 4, osch.CONTINUOUS)[0] == 110
    assert osch.timeline([10] * 6, [30] * 6, 4, osch.CONTINUOUS)[0] == 60
    rnd = random.Random(11)
    checked = {"one": 0, "copy": 0, "compute": 0}
    for _ in range(3000):
        L = rnd.randint(2, 24)
        N = rnd.randint(1, L)
        c, x = rnd.randint(1, 20), rnd.randint(0, 200)
        K, r = L // N, L % N
        T = osch.timeline([c] * L, [x] * L, N, osch.CONTINUOUS)[0]
        if K == 1:
            assert T == max(L * c, x + c)
            checked["one"] += 1
        elif x >= (2 * N + r) * c:                   # copy stream never idles: the analyzer's regime (Sec. 4.4)
            assert T == K * x
            checked["copy"] += 1
        elif x + c <= 2 * N * c and K * x <= L * c:  # every load is back before its layer is reached
            assert T == L * c
            checked["compute"] += 1
    assert min(checked.values()) > 100
    for _ in range(300):
        L = rnd.randint(1, 12)
        N = rnd.randint(1, L + 1)
        tc = [rnd.randint(1, 100) for _ in range(L)]
        tx = [rnd.randint(0, 600) for _ in range(L)]
        times, _ = osch.timeline_continuous(tc, tx, N, 6)
        assert times == _dependency_graph_times(tc, tx, N, 6), (tc, tx, N)
        assert times[0] == osch.timeline(tc, tx, N, osch.EAGER)[0]          # a cold start is the eager schedule
        steady = osch.timeline(tc, tx, N, osch.CONTINUOUS)[0]
        assert max(sum(tc), sum(tx[o] for o in osch.offloaded_layers(L, N))) <= steady <= times[0]
        assert steady == max(osch.timeline_continuous(tc, tx, N, 40)[0][-2:])   # 16 iterations reach the steady state
    # the repaired closed form of Sec. 4.4 is this schedule's answer whenever the copy stream is the
    # bottleneck: the SLO admits floor(SLO / x) transfers per iteration
    L, c, x = 32, 10, 830
    for slo in (2 * L * c, 3 * L * c, 5 * L * c, 10 * L * c):
        n = osch.min_interval([c] * L, [x] * L, slo, osch.CONTINUOUS)
        k_allowed = slo // x
        assert (L // n if n <= L else 0) <= k_allowed
        assert n == osch.paper_rule(L, c, x, slo) or x + c > slo   # K = 1 costs x + c, not x


def test_picker_is_min_feasible_and_monotone_in_slo():
    rnd = random.Random(3)
    for _ in range(400):
        L = rnd.randint(1, 16)
        tc = [rnd.randint(1, 100) for _ in range(L)]
        tx = [rnd.randint(0, 600) for _ in range(L)]
        prev = None
        for slo in sorted(rnd.randint(1, 4000) for _ in range(8)):
            n = osch.min_interval(tc, tx, slo)
            feas = [N for N in range(1, L + 1) if osch.timeline(tc, tx, N)[0] <= slo]
            if feas:
                assert n == min(feas)
            elif sum(tc) <= slo:
                assert n == L + 1
            else:
                assert n is None
            if prev is not None:            # a looser SLO never needs a larger interval
                assert n is not None and n <= prev
            prev = n if n is not None else prev


def test_pick_respects_capacity():
    tc, tx = [10] * 8, [35] * 8
    # T(N): N=1: 35+7*35+10=290; N=2: 80+4*25=180; N=3: 80+2*15=110; N=4: 80+2*5=90; N>=5: 80
    assert [osch.timeline(tc, tx, N)[0] for N in range(1, 10)] == [290, 180, 110, 90, 80, 80, 80, 80, 80]
    assert osch.min_interval(tc, tx, 100) == 4
    assert osch.pick_interval(tc, tx, 100, n_max=9) == 4
    assert osch.pick_interval(tc, tx, 100, n_max=4) == 4
    assert osch.pick_interval(tc, tx, 100, n_max=3) is None       # minimum > maximum: reject
    assert osch.pick_interval(tc, tx, 79, n_max=9) is None        # below the un-offloaded time
    assert osch.pick_interval(tc, tx, 80, n_max=9) == 5
    assert osch.min_interval([10] * 4, [100] * 4, 40) == 5         # only "offload nothing" meets it


def test_capacity_bound():
    L, state, slot, fixed = 8, 100, 100, 50
    # R(N) = (L-K)*100 + 200 (if K) + 50
    assert osch.resident_bytes(L, 1, state, slot, fixed) == 250
    assert osch.resident_bytes(L, 2, state, slot, fixed) == 650
    assert osch.resident_bytes(L, 8, state, slot, fixed) == 950
    assert osch.resident_bytes(L, 9, state, slot, fixed) == 850   # nothing offloaded: no slots
    assert osch.max_interval(L, 250, state, slot, fixed) == 1
    assert osch.max_interval(L, 249, state, slot, fixed) == 0
    assert osch.max_interval(L, 700, state, slot, fixed) == 2
    assert osch.max_interval(L, 850, state, slot, fixed) == 9     # model fits: no upper limit
    assert osch.max_interval(L, 0, state, slot, fixed) == 9
    prev = 0
    for N in range(1, L + 1):
        r = osch.resident_bytes(L, N, state, slot, fixed)
        assert r >= prev
        prev = r


def test_max_tokens_hand_worked():
    """Sec. 5.6 / Fig. 14: a smaller interval frees GPU memory for tokens.  L = 8 layers of 100 B of
    weights, 2 B of KV per token per layer, 50 B of workspace, 2050 B of GPU memory.
    Nothing offloaded: 8 states -> 8 (100 + 2t) + 50 <= 2050 -> t <= 75.
    N = 2: 4 resident + 2 slots = 6 states -> 6 (100 + 2t) <= 2000 -> t <= 116 (2t <= 233.3).
    N = 1: 2 slots only -> 2 (100 + 2t) <= 2000 -> t <= 450.
    N = 8: 7 resident + 2 slots = 9 states -> 9 (100 + 2t) <= 2000 -> t <= 61 (2t <= 122.2)."""
    args = dict(weight_bytes=100, kv_token_bytes=2, fixed_bytes=50, budget=2050)
    assert osch.max_tokens(8, 9, **args) == 75
    assert osch.max_tokens(8, 2, **args) == 116
    assert osch.max_tokens(8, 1, **args) == 450
    assert osch.max_tokens(8, 8, **args) == 61
    assert osch.max_tokens(8, 9, weight_bytes=100, kv_token_bytes=2, fixed_bytes=50, budget=849) == 0   # weights alone do not fit
    assert osch.max_tokens(8, 9, weight_bytes=100, kv_token_bytes=2, fixed_bytes=50, budget=850) == 0
    assert osch.max_tokens(8, 9, weight_bytes=100, kv_token_bytes=2, fixed_bytes=50, budget=866) == 1
    # consistent with the capacity bound: at that many tokens the interval fits, with one more it does not
    rnd = random.Random(9)
    for _ in range(300):
        L, N = rnd.randint(1, 40), rnd.randint(1, 41)
        wb, kt, fx = rnd.randint(1, 10**9), rnd.randint(1, 10**5), rnd.randint(0, 10**9)
        budget = rnd.randint(0, 60 * 10**9)
        t = osch.max_tokens(L, N, wb, kt, fx, budget)
        st = wb + t * kt
        if t > 0:
            assert osch.resident_bytes(L, N, st, st, fx) <= budget
        if osch.resident_bytes(L, N, wb, wb, fx) <= budget:
            assert osch.resident_bytes(L, N, st + kt, st + kt, fx) > budget
    # fewer resident layers never hold fewer tokens (K is non-increasing in N; the slots cost two states)
    for N in range(2, 9):
        assert osch.max_tokens(8, N, **args) >= osch.max_tokens(8, N + 1, **args) or N == 8


def _inventory(L, N, w, kv, fixed, what):
    """What the GPU holds, item by item: each layer's weights and KV slice if they live there, the
    two staging slots' parts if any layer is host-resident, the workspace."""
    items = [fixed]
    any_host = False
    for l in range(L):
        host = 1 <= N <= L and (l + 1) % N == 0
        any_host |= host
        if not host or what == osch.KV:
            items.append(w)                 # weights on the GPU
        if not host or what == osch.WEIGHTS:
            items.append(kv)                # KV slice on the GPU
    if any_host:
        for _slot in range(2):
            if what != osch.KV:
                items.append(w)
            if what != osch.WEIGHTS:
                items.append(kv)
    return sum(items)


def test_what_is_offloaded_hand_worked_and_inventory():
    """Host-resident layers may keep their whole state, only their weights or only their KV slice on the
    host.  L = 8, N = 2 (4 layers on the host), weights 100 B, KV slice 30 B, workspace 50 B:
    whole state: 4 x 130 resident + 2 slots x 130 + 50 = 830
    weights only: 4 x 130 + 4 x 30 (their KV stays) + 2 x 100 + 50 = 890
    KV only:      4 x 130 + 4 x 100 (their weights stay) + 2 x 30 + 50 = 1030;   nothing offloaded: 8 x 130 + 50 = 1090."""
    assert osch.resident_bytes_of(8, 2, 100, 30, 50, osch.STATE) == 830
    assert osch.resident_bytes_of(8, 2, 100, 30, 50, osch.WEIGHTS) == 890
    assert osch.resident_bytes_of(8, 2, 100, 30, 50, osch.KV) == 1030
    assert osch.resident_bytes_of(8, 9, 100, 30, 50, osch.KV) == 1090
    assert osch.load_bytes(100, 12, osch.STATE) == 112 and osch.load_bytes(100, 12, osch.WEIGHTS) == 100
    assert osch.load_bytes(100, 12, osch.KV) == 12 and osch.load_bytes(100, 0, osch.KV) == 0
    # max length, same numbers as the whole-state case above (2 B per token, budget 2050, workspace 50), N = 2:
    # weights only: 4 (100 + 2t) + 4 (2t) + 2 x 100 <= 2000 -> 16 t <= 1400 -> t <= 87
    # KV only:      4 (100 + 2t) + 4 x 100 + 2 (2t) <= 2000 -> 12 t <= 1200 -> t <= 100
    args = dict(weight_bytes=100, kv_token_bytes=2, fixed_bytes=50, budget=2050)
    assert osch.max_tokens(8, 2, what=osch.WEIGHTS, **args) == 87
    assert osch.max_tokens(8, 2, what=osch.KV, **args) == 100
    assert osch.max_tokens(8, 2, what=osch.STATE, **args) == osch.max_tokens(8, 2, **args) == 116
    rnd = random.Random(13)
    for _ in range(600):
        L, N = rnd.randint(1, 40), rnd.randint(0, 42)
        w, kv, fx = rnd.randint(0, 10**6), rnd.randint(0, 10**6), rnd.randint(0, 10**6)
        r = {what: osch.resident_bytes_of(L, N, w, kv, fx, what) for what in (osch.STATE, osch.WEIGHTS, osch.KV)}
        for what in r:
            assert r[what] == _inventory(L, N, w, kv, fx, what)
        assert r[osch.STATE] == osch.resident_bytes(L, N, w + kv, w + kv, fx)
        none = osch.resident_bytes_of(L, L + 1, w, kv, fx)
        assert r[osch.WEIGHTS] + r[osch.KV] == r[osch.STATE] + none          # the two halves add up
        budget = rnd.randint(0, 50 * 10**6)
        for what in r:
            n_max = osch.max_interval_of(L, budget, w, kv, fx, what)
            fits = [n for n in range(1, L + 2) if _inventory(L, n, w, kv, fx, what) <= budget]
            assert n_max == (max(fits) if fits else 0)
    for _ in range(200):                       # max length against a linear scan on small numbers
        L, N = rnd.randint(1, 12), rnd.randint(1, 13)
        w, kt, fx, budget = rnd.randint(1, 60), rnd.randint(1, 9), rnd.randint(0, 40), rnd.randint(0, 3000)
        for what in (osch.STATE, osch.WEIGHTS, osch.KV):
            t = 0
            while _inventory(L, N, w, (t + 1) * kt, fx, what) <= budget:
                t += 1
            if _inventory(L, N, w, 0, fx, what) > budget:
                t = 0
            assert osch.max_tokens(L, N, w, kt, fx, budget, what) == t


def test_refine_interval_hand_worked_closed_form_and_properties():
    """Intervals that offload equally many layers (same floor(L / N): same host memory, Sec. 4.3) ranked by iteration
    time.  Hand-worked: L = 8, c = 10.  With x = 65, T(N) = 80 + K max(0, 65 - 10 (N - 1)) under Fig. 7's schedule: one
    offloaded layer for N = 5..8 with T = 105, 95, 85, 80, two for N = 3, 4 with T = 170, 150.  With x = 35 nothing
    stalls from N = 5 on (35 <= 40): a tie, and the smallest interval stays."""
    tc = [10] * 8
    assert [osch.timeline(tc, [65] * 8, N)[0] for N in range(3, 9)] == [170, 150, 105, 95, 85, 80]
    assert osch.refine_interval(tc, [65] * 8, 5) == 8
    assert osch.refine_interval(tc, [65] * 8, 6) == 8
    assert osch.refine_interval(tc, [65] * 8, 3) == 4
    assert osch.refine_interval(tc, [65] * 8, 8) == 8
    assert osch.refine_interval(tc, [65] * 8, 9) == 9            # nothing offloaded: unchanged
    assert osch.refine_interval(tc, [35] * 8, 5) == 5            # tie: the smallest
    assert osch.refine_interval(tc, [45] * 8, 5) == 6            # 45 <= 10 (N - 1) first holds at N = 6
    # closed form for uniform times (N >= 2): T(N) = L c + K max(0, x - (N - 1) c) does not rise with N while K stays,
    # so the answer is the first interval of the equal-K range without a stall, else the range's last
    rnd = random.Random(23)
    for _ in range(1500):
        L = rnd.randint(2, 40)
        c, x = rnd.randint(1, 50), rnd.randint(0, 900)
        N = rnd.randint(2, L)
        K = L // N
        last = L // K                                             # largest interval that still offloads K layers
        no_stall = [n for n in range(N, last + 1) if x <= (n - 1) * c]
        assert osch.refine_interval([c] * L, [x] * L, N) == (no_stall[0] if no_stall else last)
    # measured times: the result offloads what N offloads, is never slower than N and than any interval of its range,
    # and is idempotent; the eager schedule never stalls longer, the continuous one is a steady state (both just run)
    for _ in range(600):
        L = rnd.randint(1, 24)
        tc = [rnd.randint(1, 300) for _ in range(L)]
        tx = [rnd.randint(0, 2500) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        for sched in (osch.PAPER, osch.EAGER, osch.CONTINUOUS):
            r = osch.refine_interval(tc, tx, N, sched)
            assert r >= N and (L // r if r <= L else 0) == (L // N if N <= L else 0)
            t_r = osch.timeline(tc, tx, r, sched)[0]
            same_k = [n for n in range(1, L + 1) if n >= N and L // n == L // N] if N <= L else [N]
            assert t_r == min(osch.timeline(tc, tx, n, sched)[0] for n in same_k)
            assert r == min(n for n in same_k if osch.timeline(tc, tx, n, sched)[0] == t_r)
            assert osch.refine_interval(tc, tx, r, sched) == r
            for slo in (t_r, osch.timeline(tc, tx, N, sched)[0]):   # whatever N meets, the result meets
                assert t_r <= slo or osch.timeline(tc, tx, N, sched)[0] > slo


def test_paper_rule_never_exceeds_timeline_pick():
    rnd = random.Random(4)
    for _ in range(5000):
        L, c, x = rnd.randint(1, 80), rnd.randint(1, 500), rnd.randint(1, 60000)
        slo = rnd.randint(L * c, 4 * L * c)
        n_paper = osch.paper_rule(L, c, x, slo)
        assert len(osch.offloaded_layers(L, n_paper)) <= slo // x
        if n_paper > 1:
            assert len(osch.offloaded_layers(L, n_paper - 1)) > slo // x
        n_pick = osch.min_interval([c] * L, [x] * L, slo)
        assert n_pick is not None and n_paper <= n_pick


def test_printed_formula_breaks_in_the_papers_own_regime():
    # Sec. 3.2: a layer's transfer is 13.8x its compute in decoding; delta = 50 %
    assert osch.paper_rule_as_printed(32, 1000, 13800, 1, 2) is None
    assert osch.paper_rule_as_printed(32, 1000, 300, 1, 2) == 32 // 5


def test_table1_shape(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "table1_record.txt"))
            if l.strip() and not l.startswith("#")]
    seqs = [int(v) for v in rows[0][1:]]
    table = {int(r[0]): [int(v) for v in r[1:]] for r in rows[1:]}
    batches = sorted(table)
    # the printed record: non-increasing along both axes, ends at 1
    for b in batches:
        assert table[b] == sorted(table[b], reverse=True)
    for j in range(len(seqs)):
        col = [table[b][j] for b in batches]
        assert col == sorted(col, reverse=True)
    assert table[batches[-1]][-1] == 1
    # the picker has the same shape when layer compute grows with batch*seq and the transfer is fixed
    L, x = 32, 150_000
    for delta_pct in (20, 50, 100):
        ours = {}
        for b, s in itertools.product(batches, seqs):
            c = 2_000 + 3 * b * s
            slo = L * c * (100 + delta_pct) // 100
            ours[(b, s)] = osch.min_interval([c] * L, [x] * L, slo)
        for b in batches:
            r = [ours[(b, s)] for s in seqs]
            assert r == sorted(r, reverse=True)
        for s in seqs:
            r = [ours[(b, s)] for b in batches]
            assert r == sorted(r, reverse=True)
        assert ours[(batches[-1], seqs[-1])] == 1       # compute of a layer exceeds its transfer
