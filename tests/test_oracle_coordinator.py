"""Pins of the oracle's bandwidth coordinator (oracle/coordinator.py, paper Sec. 4.5 / Fig. 8) and exact
agreement of the library's coordinator (include/sn_coord.h) with it.  CPU only."""
import random

import pytest

from oracle import coordinator as oc
from paper_2502_08182_amd import sn
from paper_2502_08182_amd import sn_coord as C

S = 1_000_000_000      # one second in ns: rates below are then simply K(N) * mem_per_layer


def test_layers_bytes_and_rate():
    g = oc.Instance(n_layers=8, mem_per_layer=100, iter_ns=S, n_min=1, n_max=9)
    assert [oc.offloaded(g, N) for N in range(1, 10)] == [8, 4, 2, 2, 1, 1, 1, 1, 0]
    assert [oc.rate(g, N) for N in (1, 2, 3, 8, 9)] == [800, 400, 200, 100, 0]
    # 3 offloaded layers of 1000 bytes every 7 ns: 3000 / 7e-9 = 428571428571.43 B/s, rounded down
    h = oc.Instance(n_layers=3, mem_per_layer=1000, iter_ns=7, n_min=1, n_max=4)
    assert oc.rate(h, 1) == 428_571_428_571 and oc.host_bytes(h, 1) == 3000 and oc.rate(h, 4) == 0


def test_two_instances_hand_worked():
    # A: L = 8, 100 B per layer: rate 800, 400, 200, 200, 100, 100, 100, 100, 0 for N = 1..9
    # B: L = 4, 300 B per layer: rate 1200, 600, 300, 300, 0 for N = 1..5         (1 s iterations)
    A = oc.Instance(8, 100, S, 1, 9)
    B = oc.Instance(4, 300, S, 1, 5)
    # link 1000 B/s, strict: (2,2) = 1000 is out.  800 B of host memory is the most: (1,5) and (3,2), both at
    # 800 B/s -> the lexicographically smaller tuple
    assert oc.adjust([A, B], 1000) == ((1, 5), 800, 800)
    # B must offload (its model does not fit: max interval 4): (1, anything) needs >= 1100 -> (3,2)
    B4 = oc.Instance(4, 300, S, 1, 4)
    assert oc.adjust([A, B4], 1000) == ((3, 2), 800, 800)
    # one byte per second more and (2,2) becomes valid: 400 + 600 = 1000 B on the host
    assert oc.adjust([A, B4], 1001) == ((2, 2), 1000, 1000)
    # B's request needs interval >= 3 for its SLO: best is A = 2 (400) + B = 3 (300)
    B3 = oc.Instance(4, 300, S, 3, 4)
    assert oc.adjust([A, B3], 1000) == ((2, 3), 700, 700)
    # not even the largest intervals fit the link: A = 8 (100) + B = 4 (300) = 400 is not < 400
    A8 = oc.Instance(8, 100, S, 1, 8)
    assert oc.adjust([A8, B4], 400) is None
    assert oc.adjust([A8, B4], 401) == ((5, 3), 400, 400)


def test_idle_neighbour_and_rejection():
    # alone on the bus (Sec. 4.5, "special case"): the request is served with its minimum interval
    g = oc.Instance(8, 100, S, 3, 9)
    assert oc.adjust([g], 10**9) == ((3,), 200, 200)
    # minimum above maximum: the SLO cannot be met within capacity -> back to the scheduler
    assert oc.adjust([oc.Instance(8, 100, S, 5, 4)], 10**9) is None
    assert oc.adjust([g, oc.Instance(8, 100, S, 5, 4)], 10**9) is None
    # a model that fits entirely may stop offloading when the link is taken
    assert oc.adjust([g], 50) == ((9,), 0, 0)
    assert oc.adjust([g], 0) is None                                   # 0 < 0 is false


def test_ties_prefer_less_bandwidth():
    # one layer each, same bytes; B iterates half as often, so it costs half the bandwidth
    A = oc.Instance(1, 100, S, 1, 2)
    B = oc.Instance(1, 100, 2 * S, 1, 2)
    assert oc.adjust([A, B], 1000) == ((1, 1), 200, 150)
    assert oc.adjust([A, B], 120) == ((2, 1), 100, 50)                 # (1,2) holds as much but costs 100 B/s
    assert oc.adjust([A, B], 50) == ((2, 2), 0, 0)


# ---- the library against the oracle -----------------------------------------------------------------

def _lib_adjust(insts, bw):
    try:
        return C.sn_coord_adjust([C.make_instance(g.n_layers, g.mem_per_layer, g.iter_ns, g.n_min, g.n_max)
                                  for g in insts], bw)
    except sn.SnError as e:
        assert e.code == sn.SN_E_INFEASIBLE
        return None


def test_library_agrees_with_the_oracle_on_the_pins():
    A, B4 = oc.Instance(8, 100, S, 1, 9), oc.Instance(4, 300, S, 1, 4)
    for bw in (0, 1, 400, 401, 700, 701, 1000, 1001, 5000):
        assert _lib_adjust([A, B4], bw) == oc.adjust([A, B4], bw), bw
    g = C.make_instance(8, 100, S, 1, 9)
    assert [C.sn_coord_offloaded(g, N) for N in range(0, 11)] == [0, 8, 4, 2, 2, 1, 1, 1, 1, 0, 0]
    assert C.sn_coord_rate(C.make_instance(3, 1000, 7, 1, 4), 1) == 428_571_428_571
    assert C.sn_coord_host_bytes(g, 2) == 400


def test_library_agrees_with_the_oracle_on_random_buses():
    rng = random.Random(5)
    for case in range(400):
        n = rng.randint(1, 4)
        insts = []
        for _ in range(n):
            L = rng.randint(1, 12)
            n_min = rng.randint(1, L + 1)
            n_max = rng.choice([L + 1, L + 1, L + 5, rng.randint(1, L + 1)])
            mem = rng.choice([1, 10, 403_000_000, rng.randint(1, 3_000_000_000)])
            it = rng.choice([S, 3, rng.randint(1_000_000, 80_000_000)])
            insts.append(oc.Instance(L, mem, it, n_min, n_max))
        peak = sum(oc.rate(g, min(g.n_min, g.n_layers)) for g in insts)
        for bw in {0, 1, peak // 3, peak // 2, peak, peak + 1, 64_000_000_000}:
            assert _lib_adjust(insts, bw) == oc.adjust(insts, bw), (case, insts, bw)


def test_library_handles_eight_instances_and_bad_arguments():
    insts = [oc.Instance(32, 403_000_000, 70_000_000, 3, 33) for _ in range(8)]
    bw = 57_000_000_000
    got = _lib_adjust(insts, bw)
    assert got is not None and got[2] < bw and all(3 <= N <= 33 for N in got[0])
    # nothing with more host memory is valid: moving any one instance to the next denser interval breaks the link
    for i in range(8):
        if got[0][i] > 3:
            denser = max(N for N in range(3, got[0][i]) if oc.offloaded(insts[i], N) > oc.offloaded(insts[i], got[0][i]))
            r = got[2] - oc.rate(insts[i], got[0][i]) + oc.rate(insts[i], denser)
            assert not r < bw
    with pytest.raises(sn.SnError) as e:
        C.sn_coord_adjust([C.make_instance(0, 1, 1, 1, 1)], 10)
    assert e.value.code == sn.SN_E_INVAL
    with pytest.raises(sn.SnError) as e:
        C.sn_coord_adjust([C.make_instance(4, 1, 0, 1, 5)], 10)
    assert e.value.code == sn.SN_E_INVAL
    with pytest.raises(sn.SnError) as e:
        C.sn_coord_adjust([C.make_instance(4, 1, 1, 1, 5)] * 9, 10)
    assert e.value.code == sn.SN_E_INVAL
