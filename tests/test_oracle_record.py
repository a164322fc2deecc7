"""Pins of the oracle's performance record (oracle/record.py, paper Sec. 4.4, Table 1) and
exact agreement of the library's record (include/sn_record.h) with it.  CPU only."""
import os
import random

import numpy as np
import pytest

from oracle import record as orec
from oracle import schedule as osch
from paper_2502_08182_amd import sn
from paper_2502_08182_amd import sn_record as R

DEC, PRE = orec.DECODE, orec.PREFILL
ABS, REL = orec.SLO_ABS_NS, orec.SLO_REL_PERMILLE


# ---- hand-worked cell: L = 4, compute 10 per layer, transfer x per layer --------------------------
# Closed forms for uniform times (Sec. 4.3's schedule): T(N) = L c + K max(0, x - (N-1) c) for
# N >= 2, T(1) = x + (L-1) max(c, x) + c.   With c = 10:
#   x = 25:  T(1) = 110, T(2) = 40 + 2*15 = 70, T(3) = 40 + 5 = 45, T(4) = 40, none = 40
#   x = 12:  T(1) = 12 + 36 + 10 = 58, T(2) = 40 + 2*2 = 44, T(3) = 40, T(4) = 40
#   x = 45:  T(1) = 45 + 135 + 10 = 190, T(2) = 40 + 2*35 = 110, T(3) = 40 + 25 = 65, T(4) = 40 + 15 = 55
def _cell(x, c=10, L=4):
    return [c] * L, [x] * L


def _hand_record(step=0):
    r = orec.Record(4, step)
    r.put(DEC, 4, 128, *_cell(45), n_max=5)
    r.put(DEC, 4, 256, *_cell(25), n_max=5)
    r.put(DEC, 8, 128, *_cell(25), n_max=5)
    r.put(DEC, 8, 256, *_cell(12), n_max=5)
    return r


def test_hand_worked_cells():
    r = _hand_record()
    # exact cells
    assert r.cell_interval(DEC, 4, 256, ABS, 70) == 2
    assert r.cell_interval(DEC, 4, 256, ABS, 69) == 3
    assert r.cell_interval(DEC, 4, 256, ABS, 45) == 3
    assert r.cell_interval(DEC, 4, 256, ABS, 44) == 4
    assert r.cell_interval(DEC, 4, 256, ABS, 40) == 4
    assert r.cell_interval(DEC, 4, 256, ABS, 39) is None
    assert r.cell_interval(DEC, 8, 256, ABS, 44) == 2
    assert r.cell_interval(DEC, 4, 128, ABS, 60) == 4
    assert r.cell_interval(DEC, 4, 128, ABS, 54) == 5          # only the un-offloaded iteration fits
    # relative bound: 1750 per mille of 40 = 70
    assert r.cell_interval(DEC, 4, 256, REL, 1750) == 2
    assert r.cell_interval(DEC, 4, 256, REL, 1749) == 3        # 69.96 -> 69
    # a stored size looks up its own cell only
    assert r.lookup(DEC, 8, 256, ABS, 44) == 2
    # between sizes: the largest interval among the four corners (45->3 at 65.., here bound 70:
    # corners ask 3 (x=45: T(3)=65), 2, 2, 1 (x=12: T(1)=58))
    assert [r.cell_interval(DEC, b, s, ABS, 70) for b, s in [(4, 128), (4, 256), (8, 128), (8, 256)]] == [3, 2, 2, 1]
    assert r.lookup(DEC, 6, 200, ABS, 70) == 3
    assert r.lookup(DEC, 6, 256, ABS, 70) == 2                 # on a grid line: two corners
    assert r.lookup(DEC, 8, 130, ABS, 70) == 2
    # below the grid: only the corners that exist
    assert r.lookup(DEC, 2, 256, ABS, 70) == 2
    assert r.lookup(DEC, 1, 1, ABS, 70) == 3
    # one corner cannot meet the bound -> neither can the query
    assert r.lookup(DEC, 6, 200, ABS, 39) is None
    # beyond the profiled range, or another phase: not answered
    for q in [(DEC, 9, 128), (DEC, 4, 257), (PRE, 4, 128)]:
        with pytest.raises(orec.NotCovered):
            r.lookup(*q, ABS, 70)


def test_refined_lookup_hand_worked():
    """Intervals 3 and 4 both keep one of the four layers on the host (floor(4 / N) = 1).  Between the sizes the lookup answers
    3; on the four corners' times T(3) = 65, 45, 45, 40 and T(4) = 55, 40, 40, 40: the slowest corner is faster at 4."""
    r = _hand_record()
    assert r.lookup(DEC, 6, 200, ABS, 70) == 3 and r.lookup_refined(DEC, 6, 200, ABS, 70) == 4
    assert r.lookup_refined(DEC, 4, 256, ABS, 45) == 4          # its own cell: T(3) = 45, T(4) = 40
    assert r.lookup_refined(DEC, 8, 256, ABS, 40) == 3          # T(3) = T(4) = 40: a tie, the smallest stays
    assert r.lookup_refined(DEC, 8, 256, ABS, 44) == 2          # two layers on the host: interval 2 is alone
    assert r.lookup_refined(DEC, 4, 128, ABS, 54) == 5          # nothing offloaded: unchanged
    assert r.lookup_refined(DEC, 6, 200, ABS, 39) is None
    with pytest.raises(orec.NotCovered):
        r.lookup_refined(DEC, 9, 128, ABS, 70)
    # a stored size reduces to the schedule's own refinement of that cell's interval
    rng = random.Random(5)
    for _ in range(200):
        L = rng.randint(1, 20)
        tc = [rng.randint(1, 300) for _ in range(L)]
        tx = [rng.randint(0, 2500) for _ in range(L)]
        rec = orec.Record(L)
        rec.put(DEC, 2, 64, tc, tx, L + 1)
        slo = rng.randint(sum(tc), 4 * sum(tc))
        n = rec.lookup(DEC, 2, 64, ABS, slo)
        assert rec.lookup_refined(DEC, 2, 64, ABS, slo) == osch.refine_interval(tc, tx, n)


def test_capacity_bound_rejects():
    r = orec.Record(4)
    r.put(DEC, 4, 128, *_cell(25), n_max=2)
    assert r.cell_interval(DEC, 4, 128, ABS, 70) == 2
    assert r.cell_interval(DEC, 4, 128, ABS, 69) is None       # needs 3 > n_max: reject (Sec. 4.5)


def test_absolute_bounds_are_rounded_down_to_the_granularity():
    r = _hand_record(step=20)
    assert r.cell_interval(DEC, 4, 256, ABS, 79) == 3          # 79 -> 60: T(2) = 70 no longer fits
    assert r.cell_interval(DEC, 4, 256, ABS, 80) == 2
    assert r.cell_interval(DEC, 4, 256, ABS, 59) == 4          # -> 40
    assert r.cell_interval(DEC, 4, 256, ABS, 39) is None       # -> 20
    assert r.cell_interval(DEC, 4, 256, REL, 1750) == 2        # relative bounds are not rounded


def test_table1_shape_from_a_compute_bound_family(golden_dir):
    """Table 1's trend: with a relative bound, larger inputs hide more transfer and need a
    smaller interval, reaching 1.  Profiles: layer compute proportional to batch x seq, transfer
    fixed; each entry is checked against the uniform closed form evaluated here independently."""
    L, x, unit, permille = 32, 4000, 1, 1200
    batches, seqs = [4, 8, 16, 32, 64], [128, 256, 512, 1024]
    r = orec.Record(L)
    for b in batches:
        for s in seqs:
            r.put(PRE, b, s, [unit * b * s] * L, [x] * L, n_max=L + 1)
    tab = r.table(PRE, REL, permille, batches, seqs)

    def closed_form(c):
        slo = L * c * permille // 1000
        def T(N):
            if N == 1:
                return x + (L - 1) * max(c, x) + c
            return L * c + (L // N) * max(0, x - (N - 1) * c)
        return next((N for N in range(1, L + 1) if T(N) <= slo), L + 1)

    for i, b in enumerate(batches):
        for j, s in enumerate(seqs):
            assert tab[i][j] == closed_form(unit * b * s), (b, s)
    a = np.array(tab)
    assert (np.diff(a, axis=0) <= 0).all() and (np.diff(a, axis=1) <= 0).all()
    assert a[-1, -1] == 1 and a[0, 0] > 1
    # the paper's printed example has the same shape (its model and SLO are not named)
    rows = [l.split() for l in open(os.path.join(golden_dir, "table1_record.txt")) if l.strip() and l[0] != "#"]
    g = np.array([[int(v) for v in row[1:]] for row in rows[1:]])
    assert (np.diff(g, axis=0) <= 0).all() and (np.diff(g, axis=1) <= 0).all() and g[-1, -1] == 1 and g[0, 0] > 1


def test_json_round_trip():
    r = _hand_record(step=2_000_000)
    r.put(PRE, 16, 512, [3, 1, 4, 1], [5, 9, 2, 6], n_max=3)
    back = orec.Record.from_json(r.to_json())
    assert back.L == r.L and back.step == r.step and back.cells == r.cells


# ---- the library's record against the oracle's ------------------------------------------------------

def _random_record(rng, L, step):
    o = orec.Record(L, step)
    c = R.sn_record_create(L, step)
    for phase in (DEC, PRE):
        bs = sorted(rng.sample([1, 2, 4, 8, 16, 32, 64], rng.randint(1, 4)))
        ss = sorted(rng.sample([64, 128, 256, 512, 1024, 2048], rng.randint(1, 4)))
        for b in bs:
            for s in ss:
                if rng.random() < 0.15:
                    continue                    # holes in the grid
                base = rng.randint(5, 400) * (b * s if phase == PRE else 1 + b * s // 64)
                tc = [max(0, base + rng.randint(-base // 4, base // 4)) for _ in range(L)]
                xb = rng.randint(1, 30) * base
                tx = [max(0, xb + rng.randint(-xb // 8, xb // 8)) for _ in range(L)]
                n_max = rng.choice([L + 1, L + 1, rng.randint(0, L + 1)])
                o.put(phase, b, s, tc, tx, n_max)
                R.sn_record_put(c, phase, b, s, tc, tx, n_max)
    return o, c


def _lib_answer(fn, *args):
    try:
        return fn(*args)
    except sn.SnError as e:
        return {sn.SN_E_INFEASIBLE: None, sn.SN_E_STATE: "not covered"}[e.code]


def test_library_record_agrees_with_the_oracle(tmp_path):
    rng = random.Random(11)
    checked = 0
    for case in range(60):
        L = rng.randint(1, 24)
        step = rng.choice([0, 0, 1000, 2_000_000])
        o, c = _random_record(rng, L, step)
        try:
            assert R.sn_record_cells(c) == len(o.cells) and R.sn_record_layers(c) == L
            if case % 10 == 0:                    # persistence: library writes, oracle reads, library re-reads
                path = str(tmp_path / f"rec{case}.json")
                R.sn_record_save(c, path)
                assert orec.Record.from_json(open(path).read()).cells == o.cells
                c2 = R.sn_record_load(path)
                R.sn_record_destroy(c)
                c = c2
                assert R.sn_record_cells(c) == len(o.cells)
            for (phase, b, s), cell in o.cells.items():
                tc, tx, n_max = R.sn_record_get(c, phase, b, s)
                assert tc.tolist() == cell["tc"] and tx.tolist() == cell["tx"] and n_max == cell["n_max"]
            for _ in range(60):
                phase = rng.choice([DEC, PRE])
                b, s = rng.randint(1, 70), rng.randint(1, 2200)
                if rng.random() < 0.4 and o.cells:
                    phase, b, s = rng.choice(list(o.cells))
                if rng.random() < 0.5:
                    kind, val = REL, rng.choice([1000, 1050, 1200, 1500, 2000, 3000, 10000, 999])
                else:
                    ref = sum(next(iter(o.cells.values()))["tc"]) if o.cells else 1000
                    kind, val = ABS, rng.randint(0, 4 * ref + 10)
                try:
                    want = o.lookup(phase, b, s, kind, val)
                except orec.NotCovered:
                    want = "not covered"
                assert _lib_answer(R.sn_record_lookup, c, phase, b, s, kind, val) == want, (case, phase, b, s, kind, val)
                try:
                    want_r = o.lookup_refined(phase, b, s, kind, val)
                except orec.NotCovered:
                    want_r = "not covered"
                assert _lib_answer(R.sn_record_lookup_refined, c, phase, b, s, kind, val) == want_r, (case, phase, b, s, kind, val)
                if (phase, b, s) in o.cells:
                    assert _lib_answer(R.sn_record_cell_interval, c, phase, b, s, kind, val) == \
                        o.cell_interval(phase, b, s, kind, val)
                checked += 1
            bs, ss = [1, 3, 8, 20, 64], [64, 100, 512, 2048]
            for phase in (DEC, PRE):
                assert R.sn_record_table(c, phase, REL, 1500, bs, ss).tolist() == o.table(phase, REL, 1500, bs, ss)
        finally:
            R.sn_record_destroy(c)
    assert checked == 3600


def test_library_record_rejects_bad_input(tmp_path):
    c = R.sn_record_create(3, 0)
    try:
        for bad in [(2, 1, 1), (0, 0, 1), (0, 1, 0)]:
            with pytest.raises(sn.SnError) as e:
                R.sn_record_put(c, *bad, [1, 1, 1], [1, 1, 1], 4)
            assert e.value.code == sn.SN_E_INVAL
        with pytest.raises(sn.SnError):
            R.sn_record_put(c, 0, 1, 1, [1, -1, 1], [1, 1, 1], 4)
        with pytest.raises(sn.SnError):
            R.sn_record_put(c, 0, 1, 1, [1, 1, 1], [1, 1, 1], 5)       # n_max beyond L + 1
        with pytest.raises(sn.SnError) as e:
            R.sn_record_get(c, 0, 1, 1)
        assert e.value.code == sn.SN_E_STATE
    finally:
        R.sn_record_destroy(c)
    with pytest.raises(sn.SnError) as e:
        R.sn_record_load(str(tmp_path / "missing.json"))
    assert e.value.code == sn.SN_E_STATE
    for i, text in enumerate(["", "{", "[]", '{"format": "x", "version": 1, "n_layers": 1, "slo_step_ns": 0, "cells": []}',
                              '{"format": "select-n performance record", "version": 1, "n_layers": 2, "slo_step_ns": 0, '
                              '"cells": [{"phase": 0, "batch": 1, "seq": 1, "n_max": 1, "tc_ns": [1], "tx_ns": [1, 2]}]}',
                              '{"format": "select-n performance record", "version": 1, "n_layers": 1, "slo_step_ns": 0, '
                              '"cells": [{"phase": 0, "batch": 1, "seq": 1, "n_max": 1, "tc_ns": [1.5], "tx_ns": [1]}]}']):
        path = tmp_path / f"bad{i}.json"
        path.write_text(text)
        with pytest.raises(sn.SnError) as e:
            R.sn_record_load(str(path))
        assert e.value.code == sn.SN_E_INVAL, text
