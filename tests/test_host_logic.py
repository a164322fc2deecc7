"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-side schedule arithmetic (placement, timeline, picker, capacity
bound, closed form) agrees exactly with the oracle.  No GPU compute is called."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

from oracle import schedule as osch
from paper_2502_08182_amd import sn, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions(header="sn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 18
    L = sn.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(sn.EXPORTS) == names          # the binding covers exactly the header
    from paper_2502_08182_amd import sn_kernels
    knames = _declared_functions("sn_kernels.h")
    for n in knames:
        assert hasattr(L, n), n
    assert sorted(sn_kernels.EXPORTS) == knames
    from paper_2502_08182_amd import sn_record
    rnames = [n for n in _declared_functions("sn_record.h") if n.startswith("sn_record_")]
    assert len(rnames) == 13
    for n in rnames:
        assert hasattr(L, n), n
    assert sorted(sn_record.EXPORTS) == rnames
    from paper_2502_08182_amd import sn_coord
    cnames = [n for n in _declared_functions("sn_coord.h") if n.startswith("sn_coord_")]
    assert len(cnames) == 4
    for n in cnames:
        assert hasattr(L, n), n
    assert sorted(sn_coord.EXPORTS) == cnames


def test_weight_tiling_is_a_permutation_with_the_documented_index():
    from paper_2502_08182_amd import sn_kernels
    N, K = 48, 96
    src = np.arange(N * K, dtype=np.uint16).reshape(N, K)
    dst = sn_kernels.sn_k_tile_weights(src, N, K)
    assert sorted(dst.tolist()) == sorted(src.reshape(-1).tolist())
    for n, k in [(0, 0), (5, 7), (17, 40), (47, 95), (31, 64), (16, 31)]:
        at = ((n // 16) * (K // 32) + k // 32) * 512 + ((n % 16) + 16 * ((k % 32) // 8)) * 8 + k % 8
        assert dst[at] == src[n, k]
    # interleaving two matrices block by block (gate / up)
    a = np.full((32, 32), 1, dtype=np.uint16)
    b = np.full((32, 32), 2, dtype=np.uint16)
    out = np.zeros(2 * 32 * 32, dtype=np.uint16)
    sn_kernels.sn_k_tile_weights(a, 32, 32, out, 2, 0)
    sn_kernels.sn_k_tile_weights(b, 32, 32, out, 2, 1)
    assert out.reshape(4, 512)[:, 0].tolist() == [1, 2, 1, 2]


def test_bf16_weights_become_equal_float16_values():
    """Every one of the 65536 bfloat16 bit patterns, against numpy's float32 -> float16 rounding."""
    from paper_2502_08182_amd import sn_kernels
    bits = np.arange(65536, dtype=np.uint16).reshape(64, 1024)
    tiled, bad = sn_kernels.sn_k_tile_weights(bits, 64, 1024, bf16_to_f16=True, return_bad=True)
    plain = sn_kernels.sn_k_tile_weights(bits, 64, 1024)            # same permutation, no conversion
    src = synth.widen(plain, "bf16")
    got = tiled.view(np.float16).astype(np.float64)
    with np.errstate(over="ignore"):
        want = src.astype(np.float32).astype(np.float16).astype(np.float64)
    fin = np.isfinite(src) & (np.abs(src) <= 65504.0)
    assert np.array_equal(got[fin], want[fin])
    exact = fin & ((np.abs(src) >= 2.0 ** -17) | (src == 0))
    assert np.array_equal(got[exact], src[exact])                    # exact, not merely nearest
    assert bad == int((~fin).sum())                                  # overflow, inf and NaN are counted
    assert np.isnan(got[np.isnan(src)]).all() and np.isinf(got[~fin & ~np.isnan(src)]).all()


def test_tiny_bf16_weights_round_to_float16_subnormals_far_below_the_bar():
    """bfloat16 weights below 2^-17 have no equal float16 value; the library rounds them to the nearest
    float16 subnormal (absolute error below 2^-25 each) instead of refusing them.  With a tenth of a
    layer's weights pushed into that range, the oracle's layer output with the converted weights differs
    from the one with the original weights by far less than the parity bar of 2e-2 x RMS."""
    from oracle import forward as ofw
    from paper_2502_08182_amd import sn_kernels
    s = synth.ModelShape(1, 256, 4, 2, 64, 512, act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16")
    rng = np.random.default_rng(17)
    layer = synth.make_layer(s, 0, 0)
    conv, worst = {}, 0.0
    for name, bits in layer.items():
        if bits.ndim == 2:
            v = synth.widen(bits, "bf16")
            tiny = rng.random(v.shape) < 0.1
            v = np.where(tiny, v * 2.0 ** -14, v)                      # N(0, 0.02) * 2^-14: mostly below 2^-17
            bits = synth.to_bits(v, "bf16")
            layer[name] = bits
            n, k = bits.shape
            tiled, bad = sn_kernels.sn_k_tile_weights(bits, n, k, bf16_to_f16=True, return_bad=True)
            assert bad == 0
            # undo the tiling: tile the element indices with the same routine (32-bit indices via two 16-bit halves)
            idx = np.arange(n * k, dtype=np.uint32).reshape(n, k)
            lo = sn_kernels.sn_k_tile_weights((idx & 0xffff).astype(np.uint16), n, k).astype(np.uint32)
            hi = sn_kernels.sn_k_tile_weights((idx >> 16).astype(np.uint16), n, k).astype(np.uint32)
            back = np.empty(n * k, dtype=np.float64)
            back[(hi << 16) | lo] = tiled.view(np.float16).astype(np.float64)
            conv[name] = back.reshape(n, k)
            src = synth.widen(bits, "bf16")
            assert (np.abs(src) < 2.0 ** -17).mean() > 0.05            # the case is really exercised
            worst = max(worst, float(np.abs(conv[name] - src).max()))
            big = np.abs(src) >= 2.0 ** -17
            assert np.array_equal(conv[name][big], src[big])
        else:
            conv[name] = synth.widen(bits, "bf16")
    assert 0.0 < worst <= 2.0 ** -25
    x = rng.standard_normal((24, s.hidden))
    outs = []
    for wts in (synth.widen_layer(s, layer), conv):
        cache = ofw.new_cache(1, 1, s.n_kv_heads, s.head_dim)
        outs.append(ofw.step(s.as_dict(), [wts], [x], cache, kv_dtype="f16")[0])
    rms = float(np.sqrt((outs[0] ** 2).mean()))
    diff = float(np.abs(outs[0] - outs[1]).max())
    print(f"tiny weights: max|d| = {diff / rms:.2e} x RMS", flush=True)
    assert diff <= 1e-5 * rms


def test_struct_sizes_match_header():
    assert ctypes.sizeof(sn.sn_model_shape) == 16 * 4
    assert ctypes.sizeof(sn.sn_step_stats) == 6 * 8 + 8 + 2 * 4 + 8 + 8 * 8 + 8 * 4 + 8     # n_preissued, nonfinite


def test_placement_matches_oracle_and_fig7():
    off, trig = sn.sn_placement(8, 4)
    assert list(np.nonzero(off)[0] + 1) == [4, 8]               # Fig. 7, layers counted from 1
    assert [int(trig[3]) + 1, int(trig[7]) + 1] == [1, 5]
    for L in range(1, 34):
        for N in range(0, L + 3):
            off, trig = sn.sn_placement(L, N)
            want = osch.offloaded_layers(L, N)
            assert list(np.nonzero(off)[0]) == want
            assert [int(trig[o]) for o in want] == osch.trigger_layers(L, N)
            assert all(int(trig[l]) == -1 for l in range(L) if not off[l])


def test_timeline_matches_oracle():
    rnd = random.Random(11)
    for _ in range(3000):
        L = rnd.randint(1, 40)
        tc = [rnd.randint(0, 5000) for _ in range(L)]
        tx = [rnd.randint(0, 40000) for _ in range(L)]
        N = rnd.randint(0, L + 2)
        T, stalls = osch.timeline(tc, tx, N)
        assert sn.sn_timeline(tc, tx, N) == (T, sum(stalls)), (tc, tx, N)


def test_picker_matches_oracle():
    rnd = random.Random(12)
    seen = {"ok": 0, "none": 0}
    for _ in range(2000):
        L = rnd.randint(1, 32)
        tc = [rnd.randint(1, 3000) for _ in range(L)]
        tx = [rnd.randint(0, 30000) for _ in range(L)]
        slo = rnd.randint(1, 3 * sum(tc))
        n_max = rnd.randint(0, L + 1)
        want = osch.pick_interval(tc, tx, slo, n_max)
        if want is None:
            with pytest.raises(sn.SnError) as e:
                sn.sn_pick_interval_from_times(tc, tx, slo, n_max)
            assert e.value.code == sn.SN_E_INFEASIBLE
            seen["none"] += 1
        else:
            assert sn.sn_pick_interval_from_times(tc, tx, slo, n_max) == want
            seen["ok"] += 1
    assert seen["ok"] > 200 and seen["none"] > 200


def test_paper_rule_matches_oracle():
    rnd = random.Random(13)
    for _ in range(2000):
        L, c, x = rnd.randint(1, 80), rnd.randint(1, 500), rnd.randint(1, 60000)
        slo = rnd.randint(1, 4 * L * c)
        assert sn.sn_paper_rule(L, x, slo) == osch.paper_rule(L, c, x, slo)


def test_bad_arguments_are_errors_not_crashes():
    with pytest.raises(sn.SnError) as e:
        sn.sn_timeline([1, 2], [-1, 0], 1)
    assert e.value.code == sn.SN_E_INVAL
    with pytest.raises(sn.SnError):
        sn.sn_pick_interval_from_times([1], [-5], 10, 2)
    bad = sn.make_shape(synth.workload("c1").shape, 2, 40)
    bad.head_dim = 48
    assert sn.sn_layer_blob_bytes(bad) == 0
    with pytest.raises(sn.SnError) as e:
        sn.sn_init(bad)
    assert e.value.code == sn.SN_E_INVAL and "head_dim" in str(e.value)


def test_blob_layout_matches_generator():
    for name in ("c1", "c2t", "c3t", "c5t"):
        w = synth.workload(name)
        _, total = synth.blob_layout(w.shape)
        assert sn.sn_layer_blob_bytes(sn.make_shape(w.shape, 2, 64)) == total


def test_init_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(sn.SnError) as e:
        sn.sn_init(sn.make_shape(synth.workload("c1").shape, 2, 40))
    assert e.value.code == sn.SN_E_HIP


def test_max_tokens_agrees_with_the_oracle():
    """Sec. 5.6's max length: the library's closed form against the oracle's search from the definition."""
    assert sn.sn_max_tokens(8, 2, 100, 2, 50, 2050) == 116 and sn.sn_max_tokens(8, 0, 100, 2, 50, 2050) == 75
    rnd = random.Random(12)
    for _ in range(2000):
        L, N = rnd.randint(1, 80), rnd.randint(1, 82)
        wb, kt, fx = rnd.randint(1, 3 * 10**9), rnd.randint(1, 10**6), rnd.randint(0, 10**10)
        budget = rnd.choice([0, rnd.randint(0, 300 * 10**9)])
        assert sn.sn_max_tokens(L, N, wb, kt, fx, budget) == osch.max_tokens(L, N, wb, kt, fx, budget)


def test_eager_schedule_agrees_with_the_oracle():
    """Triggers, timeline and picker of the eager schedule (loads issued as early as the two staging
    slots allow) against the oracle, exactly; and never slower than the paper's schedule."""
    rnd = random.Random(31)
    for _ in range(1500):
        L = rnd.randint(1, 40)
        tc = [rnd.randint(1, 400) for _ in range(L)]
        tx = [rnd.randint(0, 3000) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        off, trig = sn.sn_placement_sched(L, N, sn.SN_SCHED_EAGER)
        want = dict(zip(osch.offloaded_layers(L, N), osch.trigger_layers(L, N, osch.EAGER)))
        assert {l: int(trig[l]) for l in range(L) if off[l]} == want
        t_o, stalls = osch.timeline(tc, tx, N, osch.EAGER)
        assert sn.sn_timeline_sched(tc, tx, N, sn.SN_SCHED_EAGER) == (t_o, sum(stalls))
        assert sn.sn_timeline_sched(tc, tx, N, sn.SN_SCHED_PAPER) == sn.sn_timeline(tc, tx, N)
        assert t_o <= sn.sn_timeline(tc, tx, N)[0]
        slo = rnd.randint(1, 3 * sum(tc))
        want_n = osch.pick_interval(tc, tx, slo, L + 1, osch.EAGER)
        try:
            got_n = sn.sn_pick_interval_from_times_sched(tc, tx, slo, L + 1, sn.SN_SCHED_EAGER)
        except sn.SnError as e:
            assert e.code == sn.SN_E_INFEASIBLE
            got_n = None
        assert got_n == want_n
    with pytest.raises(sn.SnError):
        sn.sn_timeline_sched([1], [1], 1, 3)


def test_refine_interval_agrees_with_the_oracle():
    """sn_refine_interval_from_times (the fastest of the intervals that offload as many layers as N) against the oracle,
    exactly, for the three schedules; bad arguments are errors."""
    rnd = random.Random(29)
    for _ in range(1200):
        L = rnd.randint(1, 40)
        tc = [rnd.randint(1, 400) for _ in range(L)]
        tx = [rnd.randint(0, 3000) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        for mine, theirs in ((sn.SN_SCHED_PAPER, osch.PAPER), (sn.SN_SCHED_EAGER, osch.EAGER), (sn.SN_SCHED_CONTINUOUS, osch.CONTINUOUS)):
            assert sn.sn_refine_interval_from_times(tc, tx, N, mine) == osch.refine_interval(tc, tx, N, theirs)
    assert sn.sn_refine_interval_from_times([10] * 8, [65] * 8, 5) == 8
    for bad in ((0, 0), (10, 0), (3, 7)):
        with pytest.raises(sn.SnError):
            sn.sn_refine_interval_from_times([10] * 8, [65] * 8, bad[0], bad[1])
    with pytest.raises(sn.SnError):
        sn.sn_refine_interval_from_times([10, -1], [5, 5], 1)


def test_continuous_schedule_agrees_with_the_oracle():
    """Loads that run on across the iteration boundary: steady-state iteration time, the stalls of the
    last iteration and the picker against the oracle, exactly; triggers inside an iteration are the
    eager schedule's; the steady state is never slower than a cold start."""
    rnd = random.Random(37)
    for _ in range(1200):
        L = rnd.randint(1, 40)
        tc = [rnd.randint(1, 400) for _ in range(L)]
        tx = [rnd.randint(0, 3000) for _ in range(L)]
        N = rnd.randint(1, L + 1)
        assert [list(v) for v in sn.sn_placement_sched(L, N, sn.SN_SCHED_CONTINUOUS)] == \
               [list(v) for v in sn.sn_placement_sched(L, N, sn.SN_SCHED_EAGER)]
        t_o, stalls = osch.timeline(tc, tx, N, osch.CONTINUOUS)
        assert sn.sn_timeline_sched(tc, tx, N, sn.SN_SCHED_CONTINUOUS) == (t_o, sum(stalls))
        assert t_o <= sn.sn_timeline_sched(tc, tx, N, sn.SN_SCHED_EAGER)[0]
        slo = rnd.randint(1, 3 * sum(tc))
        want_n = osch.pick_interval(tc, tx, slo, L + 1, osch.CONTINUOUS)
        try:
            got_n = sn.sn_pick_interval_from_times_sched(tc, tx, slo, L + 1, sn.SN_SCHED_CONTINUOUS)
        except sn.SnError as e:
            assert e.code == sn.SN_E_INFEASIBLE
            got_n = None
        assert got_n == want_n


def test_capacity_accounting_by_offloaded_part_agrees_with_the_oracle():
    """Footprint and max length when host-resident layers keep their whole state, only their weights or
    only their KV slice on the host: library = oracle, exactly."""
    rnd = random.Random(41)
    parts = {sn.SN_OFFLOAD_STATE: osch.STATE, sn.SN_OFFLOAD_WEIGHTS: osch.WEIGHTS, sn.SN_OFFLOAD_KV: osch.KV}
    for _ in range(1500):
        L, N = rnd.randint(1, 96), rnd.randint(0, 98)
        wb, kvb, fx = rnd.randint(0, 3 * 10**9), rnd.randint(0, 3 * 10**9), rnd.randint(0, 10**10)
        kt = rnd.randint(1, 10**6)
        budget = rnd.choice([0, rnd.randint(0, 300 * 10**9)])
        for what, o_what in parts.items():
            assert sn.sn_resident_bytes_part(L, N, wb, kvb, fx, what) == osch.resident_bytes_of(L, N, wb, kvb, fx, o_what)
            assert sn.sn_max_tokens_part(L, N, wb, kt, fx, budget, what) == osch.max_tokens(L, N if N else L + 1, wb, kt, fx, budget, o_what)
        assert sn.sn_max_tokens_part(L, N, wb, kt, fx, budget, sn.SN_OFFLOAD_STATE) == sn.sn_max_tokens(L, N, wb, kt, fx, budget)
    assert sn.sn_resident_bytes_part(4, 2, 1, 1, 1, 3) == 0 and sn.sn_max_tokens_part(4, 2, 1, 1, 1, 100, -1) == 0
