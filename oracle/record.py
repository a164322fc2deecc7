"""CPU oracle of the analyzer's performance record -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file.  It shares no code with the HIP path and imports nothing from it.

The performance record (Sec. 4.4, Table 1) stores, per phase (prefill / decoding kept
apart, Sec. 4.4 last paragraphs) and per (batch size, sequence length), what one profiled
iteration measured; the optimal interval of a cell for an SLO is the picker's answer on
those times (oracle.schedule.pick_interval).  Sizes that were not profiled are answered
"conservatively from the nearest combination" (Sec. 4.4).

Readings of the paper taken here (each listed in the design notes):
  * a cell keeps the measured per-layer times and its capacity bound rather than one
    interval per SLO: the interval for any SLO follows from them exactly, which is what
    "for each SLO generates a performance record" computes, and a table like Table 1 is
    `table()` for one SLO.
  * an SLO is either absolute (nanoseconds; rounded DOWN to the record's granularity,
    the paper's prototype uses 2 ms) or relative: per-mille of the cell's own iteration
    time without offloading (1500 = 1.5x, i.e. delta = 0.5 in Sec. 4.4).  Table 1's
    trend (larger inputs -> smaller interval) is the relative kind.
  * "conservatively choosing from the nearest combination": among the profiled batch
    sizes take the nearest one below-or-equal and the nearest one above-or-equal, the
    same for sequence lengths, and return the LARGEST interval (least offloading) any of
    those up to four cells asks for; if one of them cannot meet the SLO, neither can the
    query.  The upper corner must exist (a query beyond the profiled range is not
    answered); lower corners that were not profiled are skipped.

Parity pins (tests/test_oracle_record.py): Table 1's shape from a compute-bound family
of profiles, exact cells reduce to the picker, hand-worked neighbour cases, the
granularity rounding, save/load round trip.
"""
from __future__ import annotations

import json
from typing import Dict, List, Optional, Sequence, Tuple

from . import schedule

PREFILL, DECODE = 1, 0
SLO_ABS_NS, SLO_REL_PERMILLE = 0, 1


class NotCovered(Exception):
    """No profiled cell covers the query."""


class Record:
    def __init__(self, n_layers: int, slo_step_ns: int = 0):
        self.L = int(n_layers)
        self.step = int(slo_step_ns)
        self.cells: Dict[Tuple[int, int, int], dict] = {}

    # -- filling ---------------------------------------------------------------------
    def put(self, phase: int, batch: int, seq: int, tc: Sequence[int], tx: Sequence[int], n_max: int):
        assert len(tc) == self.L and len(tx) == self.L
        self.cells[(int(phase), int(batch), int(seq))] = {
            "tc": [int(v) for v in tc], "tx": [int(v) for v in tx], "n_max": int(n_max)}

    # -- one cell ----------------------------------------------------------------------
    def _slo_ns(self, cell: dict, kind: int, value: int) -> int:
        if kind == SLO_REL_PERMILLE:
            return sum(cell["tc"]) * int(value) // 1000
        slo = int(value)
        return slo - slo % self.step if self.step > 0 else slo

    def cell_interval(self, phase: int, batch: int, seq: int, kind: int, value: int) -> Optional[int]:
        """Optimal interval of a profiled cell; None = the SLO cannot be met within capacity."""
        cell = self.cells[(phase, batch, seq)]
        return schedule.pick_interval(cell["tc"], cell["tx"], self._slo_ns(cell, kind, value), cell["n_max"])

    # -- any size ----------------------------------------------------------------------
    def lookup(self, phase: int, batch: int, seq: int, kind: int, value: int) -> Optional[int]:
        batches = sorted({b for (p, b, _) in self.cells if p == phase})
        seqs = sorted({s for (p, _, s) in self.cells if p == phase})
        b_lo = max([b for b in batches if b <= batch], default=None)
        b_hi = min([b for b in batches if b >= batch], default=None)
        s_lo = max([s for s in seqs if s <= seq], default=None)
        s_hi = min([s for s in seqs if s >= seq], default=None)
        if b_hi is None or s_hi is None or (phase, b_hi, s_hi) not in self.cells:
            raise NotCovered((phase, batch, seq))
        best = 0
        for b in {b_lo, b_hi}:
            for s in {s_lo, s_hi}:
                if b is None or s is None or (phase, b, s) not in self.cells:
                    continue
                n = self.cell_interval(phase, b, s, kind, value)
                if n is None:
                    return None
                best = max(best, n)
        return best

    def lookup_refined(self, phase: int, batch: int, seq: int, kind: int, value: int) -> Optional[int]:
        """lookup(), then -- keeping the number of host-resident layers, floor(L / N), that its answer stands for
        (Sec. 4.3: the same host memory) -- the interval whose iteration is shortest on the times of the cells that
        were consulted, the longest of them counting (conservative, as the lookup itself); the smallest on a tie.
        The paper does not choose between intervals that offload equally many layers (schedule.refine_interval)."""
        n = self.lookup(phase, batch, seq, kind, value)
        if n is None or n > self.L:
            return n
        batches = sorted({b for (p, b, _) in self.cells if p == phase})
        seqs = sorted({s for (p, _, s) in self.cells if p == phase})
        bb = {max([b for b in batches if b <= batch], default=None), min(b for b in batches if b >= batch)}
        ss = {max([s for s in seqs if s <= seq], default=None), min(s for s in seqs if s >= seq)}
        cells = [self.cells[(phase, b, s)] for b in bb for s in ss if b is not None and s is not None and (phase, b, s) in self.cells]

        def worst(cand: int) -> int:
            return max(schedule.timeline(c["tc"], c["tx"], cand)[0] for c in cells)
        best_n, best_t = n, worst(n)
        for cand in range(n + 1, self.L + 1):
            if self.L // cand != self.L // n:
                break
            t = worst(cand)
            if t < best_t:
                best_n, best_t = cand, t
        return best_n

    def table(self, phase: int, kind: int, value: int, batches: Sequence[int], seqs: Sequence[int]) -> List[List[int]]:
        """Rows: batch sizes; columns: sequence lengths; entry: lookup (0 = cannot meet, -1 = not covered)."""
        out = []
        for b in batches:
            row = []
            for s in seqs:
                try:
                    n = self.lookup(phase, b, s, kind, value)
                    row.append(0 if n is None else n)
                except NotCovered:
                    row.append(-1)
            out.append(row)
        return out

    # -- persistence -------------------------------------------------------------------
    def to_json(self) -> str:
        cells = [{"phase": p, "batch": b, "seq": s, "n_max": c["n_max"], "tc_ns": c["tc"], "tx_ns": c["tx"]}
                 for (p, b, s), c in sorted(self.cells.items())]
        return json.dumps({"format": "select-n performance record", "version": 1, "n_layers": self.L,
                           "slo_step_ns": self.step, "cells": cells})

    @staticmethod
    def from_json(text: str) -> "Record":
        d = json.loads(text)
        r = Record(d["n_layers"], d["slo_step_ns"])
        for c in d["cells"]:
            r.put(c["phase"], c["batch"], c["seq"], c["tc_ns"], c["tx_ns"], c["n_max"])
        return r
