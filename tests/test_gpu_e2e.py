"""End-to-end GPU parity through the C ABI (sn_init / sn_place / sn_step / profiler /
picker) against the CPU oracle, plus the invariants the method promises:
the output does not depend on the offloading interval (bit-identical runs), the picked
interval equals the oracle's for the same measured times, error paths return codes."""
import math

import numpy as np
import pytest
import torch

from oracle import forward as ofw
from oracle import schedule as osch
from paper_2502_08182_amd import sn, synth
from paper_2502_08182_amd.runner import Session

pytestmark = pytest.mark.gpu

TOL = 2e-2      # max |delta| <= 2e-2 x RMS(oracle output): fp16/bf16 storage, fp32 accumulation


def rms(a):
    return math.sqrt(float((a ** 2).mean()))


KV_STORAGE = "f16"   # the library keeps the KV cache in float16 for both model dtypes


def oracle_run(w, layers_bits, prompt_bits, table_bits):
    s = w.shape
    layers = [synth.widen_layer(s, t) for t in layers_bits]
    return ofw.run_workload(s.as_dict(), layers, synth.widen(prompt_bits, s.dtype), w.prompt_lens,
                            synth.widen(table_bits, s.dtype), kv_dtype=KV_STORAGE)


def gpu_run(w, layers_bits, prompt_bits, table_bits, N, max_tokens=0, want_f32=False):
    with Session(w.shape, w.batch, w.max_seq, max_tokens) as se:
        se.load_synthetic_weights(layers=layers_bits)
        se.place(N)
        res = se.run_workload(w, prompt_bits, table_bits, want_f32)
        st = se.stats()
    return (*res, st) if want_f32 else (res[0], res[1], st)


def assert_close_f32(got_bits, got_f32, want, dtype, what):
    """The hidden states the kernels produce (fp32 residual stream) are within the bar; the
    16-bit output is exactly their nearest-even rounding, so elementwise it can be further
    off only by half an ulp of the output type (2^-11 |v| for f16, 2^-8 |v| for bf16) --
    for bf16 that alone reaches 2e-2 x RMS once an element exceeds 5.1 x RMS."""
    r = rms(want)
    err = float(np.abs(got_f32.astype(np.float64) - want).max())
    print(f"{what} (fp32 hidden): max|d|={err:.4e} = {err / r:.3e} x RMS ({r:.3e})", flush=True)
    assert np.isfinite(got_f32).all() and err <= TOL * r, (what, err, r)
    assert np.array_equal(synth.widen(got_bits, dtype), ofw.round_to_storage(got_f32.astype(np.float64), dtype)), what
    half_ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
    assert (np.abs(synth.widen(got_bits, dtype) - want) <= TOL * r + half_ulp * np.abs(want) * 1.01).all(), what


def assert_close(got_bits, want, dtype, what):
    got = synth.widen(got_bits, dtype)
    assert np.isfinite(got).all(), what
    err = float(np.abs(got - want).max())
    r = rms(want)
    print(f"{what}: max|d|={err:.4e} = {err / r:.3e} x RMS ({r:.3e})", flush=True)
    assert err <= TOL * r, (what, err, r)


def _inputs(w):
    layers = [synth.make_layer(w.shape, l, 0) for l in range(w.shape.n_layers)]
    return layers, synth.make_prompt(w), synth.make_decode_table(w)


@pytest.fixture(scope="module")
def c1():
    w = synth.workload("c1")
    layers, prompt, table = _inputs(w)
    pre, dec = oracle_run(w, layers, prompt, table)
    return w, layers, prompt, table, pre, dec


def test_config1_matches_oracle_at_interval_2(c1):
    w, layers, prompt, table, pre, dec = c1
    gpre, gdec, st = gpu_run(w, layers, prompt, table, 2)
    assert st["interval"] == 2 and st["n_offloaded"] == 2
    assert_close(gpre, pre, w.shape.dtype, "c1 prefill")
    for t in range(w.decode_steps):
        assert_close(gdec[t], dec[t], w.shape.dtype, f"c1 decode step {t}")


def test_output_is_bit_identical_for_every_interval(c1):
    w, layers, prompt, table, *_ = c1
    ref = gpu_run(w, layers, prompt, table, 0)                 # everything resident
    assert ref[2]["n_offloaded"] == 0 and ref[2]["h2d_bytes"] == 0
    for N in (1, 2, 3, 4):
        got = gpu_run(w, layers, prompt, table, N)
        assert got[2]["n_offloaded"] == w.shape.n_layers // N
        assert got[2]["h2d_bytes"] > 0
        assert np.array_equal(got[0], ref[0]), f"prefill differs at N={N}"
        assert np.array_equal(got[1], ref[1]), f"decode differs at N={N}"


def test_eager_schedule_changes_timing_only(c1):
    """Loads issued one group earlier (as soon as a staging slot is free) move the same bytes and give
    the same bits for every interval, also when the schedule is switched under a live placement."""
    w, layers, prompt, table, *_ = c1
    ref = gpu_run(w, layers, prompt, table, 0)
    for N in (1, 2, 3, 4):
        with Session(w.shape, w.batch, w.max_seq) as se:
            se.load_synthetic_weights(layers=layers)
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_EAGER)
            se.place(N)
            pre, dec = se.run_workload(w, prompt, table)
            st = se.stats()
            assert st["n_offloaded"] == w.shape.n_layers // N and st["h2d_bytes"] > 0
            assert np.array_equal(pre, ref[0]) and np.array_equal(dec, ref[1]), f"eager differs at N={N}"
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_PAPER)          # switched back without re-placing
            pre2, dec2 = se.run_workload(w, prompt, table)
            assert se.stats()["h2d_bytes"] == st["h2d_bytes"]
            assert np.array_equal(pre2, ref[0]) and np.array_equal(dec2, ref[1])
    with Session(w.shape, w.batch, w.max_seq) as se:
        with pytest.raises(sn.SnError) as e:
            sn.sn_set_schedule(se.ctx, 7)
        assert e.value.code == sn.SN_E_INVAL


def test_continuous_schedule_changes_timing_only(c1):
    """Loads issued across the iteration boundary (during decode, for the next iteration): same bits
    for every interval; from the second decode step on min(2, K) of an iteration's loads were issued
    during the one before; a placement change, a KV reset, a schedule change or new weights while such
    loads are in flight discard them without harm."""
    w, layers, prompt, table, *_ = c1
    L = w.shape.n_layers
    ref = gpu_run(w, layers, prompt, table, 0)
    for N in (1, 2, 3, 4):
        K = L // N
        with Session(w.shape, w.batch, w.max_seq) as se:
            se.load_synthetic_weights(layers=layers)
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_CONTINUOUS)
            se.place(N)
            se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
            pre = se.step(list(w.prompt_lens), True, prompt)
            assert se.stats()["n_preissued"] == 0
            outs = []
            for t in range(w.decode_steps):
                outs.append(se.step([1] * w.batch, False, table[t]))
                st = se.stats()
                assert st["n_preissued"] == (0 if t == 0 else min(2, K)), (N, t, st["n_preissued"])
                assert st["n_offloaded"] == K and st["h2d_bytes"] > 0
            assert np.array_equal(pre, ref[0]) and np.array_equal(np.stack(outs), ref[1]), f"continuous differs at N={N}"
            # loads for a ninth decode step are in flight now; a new request (KV reset) must not see them
            pre2, dec2 = se.run_workload(w, prompt, table)
            assert np.array_equal(pre2, ref[0]) and np.array_equal(dec2, ref[1])
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_PAPER)
            pre3, dec3 = se.run_workload(w, prompt, table)
            assert se.stats()["n_preissued"] == 0
            assert np.array_equal(pre3, ref[0]) and np.array_equal(dec3, ref[1])
    # the interval changes before every iteration, and the weights are set again in the middle
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        sn.sn_set_schedule(se.ctx, sn.SN_SCHED_CONTINUOUS)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        pre = se.step(list(w.prompt_lens), True, prompt)
        outs = []
        for t, N in enumerate([1, 1, 3, 0, 2, 2, 4, 1]):
            se.place(N)
            if t == 5:
                se.load_synthetic_weights(layers=layers)
            outs.append(se.step([1] * w.batch, False, table[t]))
        assert np.array_equal(pre, ref[0]) and np.array_equal(np.stack(outs), ref[1])


def test_weights_only_and_kv_only_offloading(c1):
    """Host-resident layers may keep only their weights or only their KV slice on the host: same bits
    for every interval and schedule; a decode step then loads exactly the part that lives on the host
    (the two parts add up to the whole state's load); the footprints add up the same way; switching
    the part between decode steps keeps the cache."""
    w, layers, prompt, table, *_ = c1
    L = w.shape.n_layers
    ref = gpu_run(w, layers, prompt, table, 0)
    parts = (sn.SN_OFFLOAD_STATE, sn.SN_OFFLOAD_WEIGHTS, sn.SN_OFFLOAD_KV)
    for N in (1, 2, 3, 4):
        moved, held = {}, {}
        for what in parts:
            with Session(w.shape, w.batch, w.max_seq) as se:
                se.load_synthetic_weights(layers=layers)
                sn.sn_set_offload_part(se.ctx, what)
                assert sn.sn_offload_part(se.ctx) == what
                se.place(N)
                for sched in (sn.SN_SCHED_PAPER, sn.SN_SCHED_CONTINUOUS):
                    sn.sn_set_schedule(se.ctx, sched)
                    pre, dec = se.run_workload(w, prompt, table)
                    assert np.array_equal(pre, ref[0]) and np.array_equal(dec, ref[1]), (N, what, sched)
                st = se.stats()
                moved[what], held[what] = st["h2d_bytes"], st["resident_bytes"]
                assert st["n_offloaded"] == L // N
                none = sn.sn_resident_bytes(se.ctx, 0)
        assert moved[sn.SN_OFFLOAD_WEIGHTS] > 0 and moved[sn.SN_OFFLOAD_KV] > 0
        assert moved[sn.SN_OFFLOAD_WEIGHTS] + moved[sn.SN_OFFLOAD_KV] == moved[sn.SN_OFFLOAD_STATE]
        assert held[sn.SN_OFFLOAD_WEIGHTS] + held[sn.SN_OFFLOAD_KV] == held[sn.SN_OFFLOAD_STATE] + none
    # prefill from empty caches: nothing to load when only the KV slice is on the host, weights otherwise
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        sn.sn_set_offload_part(se.ctx, sn.SN_OFFLOAD_KV)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        se.step(list(w.prompt_lens), True, prompt)
        st = se.stats()
        assert st["h2d_bytes"] == 0 and st["d2h_bytes"] > 0
        # the part changes under a live cache, before every decode step
        outs = []
        order = [sn.SN_OFFLOAD_WEIGHTS, sn.SN_OFFLOAD_STATE, sn.SN_OFFLOAD_KV, sn.SN_OFFLOAD_KV,
                 sn.SN_OFFLOAD_WEIGHTS, sn.SN_OFFLOAD_KV, sn.SN_OFFLOAD_STATE, sn.SN_OFFLOAD_WEIGHTS]
        for t, what in enumerate(order):
            sn.sn_set_offload_part(se.ctx, what)
            if t == 3:
                se.place(1)
            outs.append(se.step([1] * w.batch, False, table[t]))
            if what == sn.SN_OFFLOAD_WEIGHTS:
                assert se.stats()["d2h_bytes"] == 0
        assert np.array_equal(np.stack(outs), ref[1])
        with pytest.raises(sn.SnError) as e:
            sn.sn_set_offload_part(se.ctx, 5)
        assert e.value.code == sn.SN_E_INVAL


def test_replacing_between_iterations_keeps_the_cache(c1):
    """Sec. 4.2: a new interval is applied before the next iteration; live KV must move with it."""
    w, layers, prompt, table, *_ = c1
    ref = gpu_run(w, layers, prompt, table, 0)
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        pre = se.step(list(w.prompt_lens), True, prompt)
        outs = []
        for t, N in enumerate([1, 3, 0, 2, 4, 1, 0, 2]):
            se.place(N)
            outs.append(se.step([1] * w.batch, False, table[t]))
    assert np.array_equal(pre, ref[0])
    assert np.array_equal(np.stack(outs), ref[1])


def test_capacity_at_the_resonant_stride_is_laid_out_with_spare_rows(c1):
    """A per-sequence capacity whose head-to-head stride (rows x head_dim x 4 bytes) is a multiple of 2^19 + 2^12 bytes
    -- 2064 rows at head dimension 64 -- gets 8 spare rows in the layout (all attention workgroups would otherwise hit
    one memory channel in lock-step).  Nothing else changes: outputs are those of any other capacity, bit for bit, with
    KV slices on the host as well, and the capacity the caller gave is still the limit a step may fill."""
    w, layers, prompt, table, *_ = c1
    assert w.shape.head_dim == 64
    ref = gpu_run(w, layers, prompt, table, 0)
    for N in (0, 2):
        with Session(w.shape, w.batch, 2100) as se:
            se.load_synthetic_weights(layers=layers)
            se.place(N)
            se.kv_reset([2064] * w.batch)
            pre = se.step(list(w.prompt_lens), True, prompt)
            outs = [se.step([1] * w.batch, False, table[t]) for t in range(w.decode_steps)]
            assert np.array_equal(pre, ref[0]) and np.array_equal(np.stack(outs), ref[1])
            # fill the sequences up to their capacity, then one token more must be refused
            room = [2064 - (p + w.decode_steps) for p in w.prompt_lens]
            filler = synth.to_bits(np.random.default_rng(3).standard_normal((sum(room), w.shape.hidden)), w.shape.dtype)
            se.step(room, True, filler)
            with pytest.raises(sn.SnError) as e:
                se.step([1] * w.batch, False, table[0])
            assert e.value.code == sn.SN_E_INVAL


def test_weights_may_arrive_after_placement(c1):
    """A model larger than the host's pinned memory is loaded after sn_place: GPU-resident
    layers then have no host master until they are first offloaded (the master is copied
    back from the device).  Whatever the order, and whatever intervals follow, the output
    is the one of the ordinary order, bit for bit."""
    w, layers, prompt, table, *_ = c1
    ref = gpu_run(w, layers, prompt, table, 0)
    for first in (0, 2):
        with Session(w.shape, w.batch, w.max_seq) as se:
            se.place(first)
            se.load_synthetic_weights(layers=layers)
            se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
            pre = se.step(list(w.prompt_lens), True, prompt)
            outs = []
            for t, N in enumerate([3, 1, 0, 4, 2, 0, 1, 3]):
                se.place(N)
                if t == 4:      # weights replaced in place while some layers live on the host
                    se.load_synthetic_weights(layers=layers)
                outs.append(se.step([1] * w.batch, False, table[t]))
        assert np.array_equal(pre, ref[0]), f"prefill differs (first placement {first})"
        assert np.array_equal(np.stack(outs), ref[1]), f"decode differs (first placement {first})"


@pytest.mark.parametrize("name", ["c2t", "c3t", "c4t", "c5t"])
def test_truncated_real_shapes_match_oracle(name):
    w = synth.workload(name)
    layers, prompt, table = _inputs(w)
    pre, dec = oracle_run(w, layers, prompt, table)
    N = w.intervals[0]
    gpre, gdec, fpre, fdec, st = gpu_run(w, layers, prompt, table, N, want_f32=True)
    if w.shape.dtype == "f16":
        assert_close(gpre, pre, w.shape.dtype, f"{name} prefill")
    assert_close_f32(gpre, fpre, pre, w.shape.dtype, f"{name} prefill")
    for t in range(w.decode_steps):
        if w.shape.dtype == "f16":
            assert_close(gdec[t], dec[t], w.shape.dtype, f"{name} decode {t}")
        assert_close_f32(gdec[t], fdec[t], dec[t], w.shape.dtype, f"{name} decode {t}")
    ref = gpu_run(w, layers, prompt, table, 0)
    assert np.array_equal(gpre, ref[0]) and np.array_equal(gdec, ref[1])


@pytest.mark.parametrize("batch", [9, 16, 17, 33, 64, 65, 96, 128])
def test_decode_batches_spanning_row_tiles(batch):
    base = synth.workload("c1")
    shape = synth.ModelShape(2, 256, 8, 2, 64, 512, act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16")
    lens = tuple(int(v) for v in np.random.default_rng(batch).integers(1, 40, size=batch))
    w = synth.Workload("mix", shape, batch, lens, 2)
    layers, prompt, table = _inputs(w)
    pre, dec = oracle_run(w, layers, prompt, table)
    gpre, gdec, _ = gpu_run(w, layers, prompt, table, 2)
    assert_close(gpre, pre, shape.dtype, f"B={batch} prefill")
    for t in range(2):
        assert_close(gdec[t], dec[t], shape.dtype, f"B={batch} decode {t}")


@pytest.mark.parametrize("family", ["opt", "llama_gqa"])
def test_long_context_decode_splits_keys_across_workgroups(family):
    """With few (sequence, KV head) pairs and more than 512 cached keys an iteration splits each
    sequence's keys over several workgroups and merges the partial softmaxes in a second kernel
    (with the rotation / append fused into the split that owns the new position).  One sequence is
    long, one is short, one has an empty slot in the prefill batch (joins at the second chunk)."""
    if family == "opt":
        shape = synth.ModelShape(2, 256, 4, 4, 64, 512, act="gelu", norm="ln", rope=False, has_bias=True, dtype="f16")
    else:
        shape = synth.ModelShape(2, 512, 8, 2, 64, 512, act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16")
    lens = (700, 37, 513)
    w = synth.Workload("long", shape, 3, lens, 3)
    layers, prompt, table = _inputs(w)
    pre, dec = oracle_run(w, layers, prompt, table)
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in lens])
        # two prefill chunks; the third sequence contributes nothing to the first one
        o0, o1, o2 = 0, lens[0], lens[0] + lens[1]
        a = np.concatenate([prompt[o0:o0 + 400], prompt[o1:o1 + 37]])
        b = np.concatenate([prompt[o0 + 400:o0 + 700], prompt[o2:o2 + 513]])
        ga, fa = se.step([400, 37, 0], True, a, want_f32=True)
        gb, fb = se.step([300, 0, 513], True, b, want_f32=True)
        outs = [se.step([1, 1, 1], False, table[t], want_f32=True) for t in range(w.decode_steps)]
        with Session(w.shape, w.batch, w.max_seq) as ref:      # everything resident, same chunks: bit for bit
            ref.load_synthetic_weights(layers=layers)
            ref.place(0)
            ref.kv_reset([p + w.decode_steps for p in lens])
            ra = ref.step([400, 37, 0], True, a)
            rb = ref.step([300, 0, 513], True, b)
            routs = [ref.step([1, 1, 1], False, table[t]) for t in range(w.decode_steps)]
    assert np.array_equal(ga, ra) and np.array_equal(gb, rb)
    got_f = np.concatenate([fa[:400], fb[:300], fa[400:], fb[300:]])
    got_b = np.concatenate([ga[:400], gb[:300], ga[400:], gb[300:]])
    assert_close_f32(got_b, got_f, pre, shape.dtype, f"{family} long prefill")
    for t in range(w.decode_steps):
        assert np.array_equal(outs[t][0], routs[t])
        assert_close_f32(outs[t][0], outs[t][1], dec[t], shape.dtype, f"{family} long decode {t}")


def test_chunked_prefill_equals_oracle(c1):
    w, layers, prompt, table, pre, dec = c1
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        # sequence 0: 20 + 12 tokens, sequence 1: 5 + 27
        a = np.concatenate([prompt[0:20], prompt[32:37]])
        b = np.concatenate([prompt[20:32], prompt[37:64]])
        oa = se.step([20, 5], True, a)
        ob = se.step([12, 27], True, b)
        d0 = se.step([1, 1], False, table[0])
    got = np.concatenate([oa[:20], ob[:12], oa[20:], ob[12:]])
    assert_close(got, pre, w.shape.dtype, "chunked prefill")
    assert_close(d0, dec[0], w.shape.dtype, "decode after chunked prefill")


def test_profiler_and_picker_agree_with_oracle(c1):
    w, layers, *_ = c1
    L = w.shape.n_layers
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        for is_prefill in (False, True):
            tc, tx = sn.sn_profile_layers(se.ctx, L, is_prefill, 2, 32, reps=3)
            assert (tc > 0).all() and (tx > 0).all()
            print("prefill" if is_prefill else "decode", "tc", tc.tolist(), "tx", tx.tolist(), flush=True)
            n_max = sn.sn_max_interval(se.ctx)
            assert n_max == L + 1                                   # no budget: no upper limit
            base = int(tc.sum())
            for factor in (0.9, 1.0, 1.2, 1.5, 2.0, 5.0, 50.0):
                slo_ns = int(base * factor)
                want = osch.pick_interval(tc.tolist(), tx.tolist(), slo_ns, n_max)
                if want is None:
                    with pytest.raises(sn.SnError) as e:
                        sn.sn_pick_interval(se.ctx, slo_ns / 1e6)
                    assert e.value.code == sn.SN_E_INFEASIBLE
                else:
                    assert sn.sn_pick_interval(se.ctx, slo_ns / 1e6) == want
                    assert sn.sn_timeline(tc, tx, want)[0] <= slo_ns
                    # of the intervals that keep as many layers on the host, the fastest on these measured times
                    refined = sn.sn_refine_interval_from_times(tc, tx, want)
                    assert refined == osch.refine_interval(tc.tolist(), tx.tolist(), want)
                    assert sn.sn_refine_interval(se.ctx, want) == refined      # the same from the context's own profile
                    assert sn.sn_timeline(tc, tx, refined)[0] <= sn.sn_timeline(tc, tx, want)[0]


def test_layer_compute_time_is_deterministic_at_a_real_layer_shape():
    """The premise the method rests on (Sec. 4.3, Insight): all layers have the same structure and the same
    input size, so their compute times agree, within an iteration and from one profile to the next.  Checked
    where a layer is long enough for event timestamps to resolve it: 8 layers of the OPT-6.7B layer shape,
    decode at batch 8 over 512 cached tokens and a prefill of 4 x 256 tokens.  Within one profile the layers
    agree to a fraction of a percent; two profiles taken one after the other have been seen 6 % apart (the
    GPU's clocks move with load), which is why the benchmark keeps a guard band when it picks -- the bound
    here is 5 % across layers and 10 % between profiles."""
    import dataclasses
    s = dataclasses.replace(synth.workload("c2").shape, n_layers=8)
    L = s.n_layers
    with Session(s, 8, 520) as se:
        se.place(0)
        se.load_device_generated_weights(seed=0, distinct=1)
        for is_prefill, batch, seq in ((False, 8, 512), (True, 4, 256)):
            a, _ = sn.sn_profile_layers(se.ctx, L, is_prefill, batch, seq, reps=5)
            b, _ = sn.sn_profile_layers(se.ctx, L, is_prefill, batch, seq, reps=5)
            cv = float(np.std(a) / np.mean(a))
            drift = float(np.abs(a - b).max() / np.mean(a))
            print("prefill" if is_prefill else "decode", "tc", a.tolist(), f"cv {cv:.4f} drift between profiles {drift:.4f}", flush=True)
            assert cv < 0.05, (is_prefill, a.tolist())
            assert drift < 0.10, (is_prefill, a.tolist(), b.tolist())


def test_performance_record_profiled_on_the_gpu(c1, tmp_path):
    """The analyzer (Sec. 4.4): profile a small grid of sizes for both phases into a record, then
    every lookup must equal the oracle's record fed with the same measured times; after a
    save / load round trip too.  The picked interval is then run and its output is still the
    all-resident one."""
    from oracle import record as orec
    from paper_2502_08182_amd import sn_record as R
    w, layers, prompt, table, *_ = c1
    L = w.shape.n_layers
    ref = gpu_run(w, layers, prompt, table, 0)
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        rec = R.sn_record_create(L, 0)
        o = orec.Record(L, 0)
        try:
            wrong = R.sn_record_create(L + 1, 0)
            with pytest.raises(sn.SnError) as e:
                R.sn_record_profile(wrong, se.ctx, R.SN_PHASE_DECODE, 1, 16, 2)
            assert e.value.code == sn.SN_E_INVAL                    # layer counts differ
            R.sn_record_destroy(wrong)
            for phase in (R.SN_PHASE_DECODE, R.SN_PHASE_PREFILL):
                for b in (1, 2):
                    for s in (16, 32):
                        R.sn_record_profile(rec, se.ctx, phase, b, s, 2)
                        tc, tx, n_max = R.sn_record_get(rec, phase, b, s)
                        assert (tc > 0).all() and (tx > 0).all() and n_max == sn.sn_max_interval(se.ctx) == L + 1
                        o.put(phase, b, s, tc.tolist(), tx.tolist(), n_max)
            assert R.sn_record_cells(rec) == 8
            path = str(tmp_path / "record.json")
            R.sn_record_save(rec, path)
            rec2 = R.sn_record_load(path)
            for r in (rec, rec2):
                for phase in (R.SN_PHASE_DECODE, R.SN_PHASE_PREFILL):
                    for b, s in [(1, 16), (2, 32), (2, 20), (1, 1), (2, 24)]:
                        for permille in (1000, 1100, 1500, 3000, 20000, 900):
                            want = o.lookup(phase, b, s, orec.SLO_REL_PERMILLE, permille)
                            try:
                                got = R.sn_record_lookup(r, phase, b, s, R.SN_SLO_REL_PERMILLE, permille)
                            except sn.SnError as e:
                                assert e.code == sn.SN_E_INFEASIBLE
                                got = None
                            assert got == want, (phase, b, s, permille)
            R.sn_record_destroy(rec2)
            # separate intervals per phase (Sec. 4.4): place what each phase's record says, run, compare
            n_pre = R.sn_record_lookup(rec, R.SN_PHASE_PREFILL, 2, 32, R.SN_SLO_REL_PERMILLE, 3000)
            n_dec = R.sn_record_lookup(rec, R.SN_PHASE_DECODE, 2, 32, R.SN_SLO_REL_PERMILLE, 3000)
            print("record: prefill interval", n_pre, "decode interval", n_dec, flush=True)
            se.place(n_pre)
            se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
            pre = se.step(list(w.prompt_lens), True, prompt)
            se.place(n_dec)
            outs = [se.step([1] * w.batch, False, table[t]) for t in range(w.decode_steps)]
            assert np.array_equal(pre, ref[0]) and np.array_equal(np.stack(outs), ref[1])
        finally:
            R.sn_record_destroy(rec)


def test_budget_and_call_order_errors():
    w = synth.workload("c1")
    cs = sn.make_shape(w.shape, w.batch, w.max_seq)
    with Session(w.shape, w.batch, w.max_seq) as se:
        x = torch.zeros(2, 256, dtype=torch.int16, device="cuda")
        lens = np.zeros(2, dtype=np.int32)
        with pytest.raises(sn.SnError) as e:
            sn.sn_step(se.ctx, [1, 1], False, x, lens, x)
        assert e.value.code == sn.SN_E_STATE                       # before sn_place
        with pytest.raises(sn.SnError) as e:
            sn.sn_pick_interval(se.ctx, 1.0)
        assert e.value.code == sn.SN_E_STATE                       # before a profile
        se.place(2)
        with pytest.raises(sn.SnError) as e:
            sn.sn_step(se.ctx, [1, 1], False, x, lens, x)
        assert e.value.code == sn.SN_E_STATE                       # before sn_kv_reset
        se.kv_reset([4, 4])
        with pytest.raises(sn.SnError) as e:
            sn.sn_step(se.ctx, [5, 1], True, x, se.kv_len, x)      # over capacity
        assert e.value.code == sn.SN_E_INVAL
        with pytest.raises(sn.SnError) as e:
            sn.sn_kv_reset(se.ctx, [w.max_seq * 2, w.max_seq])
        assert e.value.code == sn.SN_E_INVAL
        full = sn.sn_resident_bytes(se.ctx, 0)
        r = [sn.sn_resident_bytes(se.ctx, N) for N in range(1, 6)]
        state = (r[1] - r[0]) // 2                                 # N=1 -> N=2 makes two more layers resident
        assert r[4] == full and r[0] == full - 2 * state          # N=1: no resident layer, two slots
        assert r[2] == r[3] == full + state                        # one offloaded layer + two slots
        assert r == sorted(r[:4]) + [full]
    # a budget that only N = 1 fits
    ctx = sn.sn_init(cs, r[0], 0)
    try:
        assert sn.sn_max_interval(ctx) == 1
        sn.sn_place(ctx, 1)
        with pytest.raises(sn.SnError) as e:
            sn.sn_place(ctx, 2)
        assert e.value.code == sn.SN_E_BUDGET
        # keeping only one part on the host leaves the other on the GPU: over this budget, refused, nothing changes
        for what in (sn.SN_OFFLOAD_WEIGHTS, sn.SN_OFFLOAD_KV):
            with pytest.raises(sn.SnError) as e:
                sn.sn_set_offload_part(ctx, what)
            assert e.value.code == sn.SN_E_BUDGET
            assert sn.sn_offload_part(ctx) == sn.SN_OFFLOAD_STATE and sn.sn_resident_bytes(ctx, 1) == r[0]
        sn.sn_set_budget_enforce(ctx, False)
        sn.sn_place(ctx, 2)                                        # over the cap, allowed when enforcement is off
        sn.sn_set_offload_part(ctx, sn.SN_OFFLOAD_KV)              # and so is this, now
        assert sn.sn_offload_part(ctx) == sn.SN_OFFLOAD_KV
        assert sn.sn_resident_bytes(ctx, 1) > r[0] and sn.sn_resident_bytes(ctx, 2) == r[1]    # 4 weights stay; 2 stay + 2 KV slots
    finally:
        sn.sn_destroy(ctx)
    ctx = sn.sn_init(cs, r[0] - 1, 0)
    try:
        assert sn.sn_max_interval(ctx) == 0
        with pytest.raises(sn.SnError) as e:
            sn.sn_place(ctx, 1)
        assert e.value.code == sn.SN_E_BUDGET
    finally:
        sn.sn_destroy(ctx)


def test_float16_overflow_of_a_hand_off_is_reported(c1):
    """Activations pass between the kernels in float16: a value beyond 65504 overflows there.  The iteration's
    statistics say so (it reaches the fp32 residual stream as inf / NaN, which the final cast checks); a healthy
    model reports nothing."""
    w, layers, prompt, table, *_ = c1
    hot = [dict(t) for t in layers]
    big = synth.widen(layers[0]["wu"], "f16") * 2.0 ** 16          # |w| ~ 1300: representable, products are not
    hot[0]["wu"] = synth.to_bits(big, "f16")
    for tensors, want in ((layers, 0), (hot, 1)):
        with Session(w.shape, w.batch, w.max_seq) as se:
            se.load_synthetic_weights(layers=tensors)
            se.place(2)
            se.kv_reset([p + 2 for p in w.prompt_lens])
            out = se.step(list(w.prompt_lens), True, prompt)
            assert se.stats()["nonfinite"] == want
            assert np.isfinite(synth.widen(out, "f16")).all() == (want == 0)
            se.step([1] * w.batch, False, table[0])
            assert se.stats()["nonfinite"] == want


def test_stall_and_hidden_fraction_are_reported(c1):
    w, layers, prompt, table, *_ = c1
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        sn.sn_set_timing(se.ctx, 2)
        se.run_workload(w, prompt, table)
        st = se.stats()
        comp, stall, h2d = sn.sn_get_layer_times(se.ctx, w.shape.n_layers)
    print(st, comp.tolist(), stall.tolist(), h2d.tolist(), flush=True)
    assert st["iter_ns"] > 0 and st["h2d_ns"] > 0 and 0.0 <= st["hidden_fraction"] <= 1.0
    assert st["h2d_bytes"] > 0 and st["h2d_bytes"] % 2 == 0 and st["n_offloaded"] == 2
    assert (comp > 0).all() and stall[0] == 0 and stall[2] == 0 and h2d[1] > 0 and h2d[3] > 0
    assert st["kernel_calls"]["ffn_up"] == w.shape.n_layers and st["kernel_ns"]["ffn_up"] > 0


def test_full_size_config2_offloaded_equals_resident_and_sampled_rows_match_oracle():
    """The OPT-6.7B-shaped configuration at full size (32 layers, batch 8, prompt 512), in the launch
    configuration bench.py times.  The whole forward is ~1e14 flop, out of the oracle's reach,
    so: (i) offloaded (N=8) and all-resident runs are bit-identical and finite for the prefill
    and two decode steps; (ii) a property that holds at any size pins the numbers to the oracle:
    with the output projections (wo, wd) and their biases zeroed in layers 2..L-1, the model
    reduces to its first TWO layers, which the oracle computes for sampled rows of the full-size
    batch (the first 40 tokens of sequence 0: causal, so they depend on nothing later)."""
    w = synth.workload("c2")
    s = w.shape
    L, B, P = s.n_layers, w.batch, 512
    rng = np.random.default_rng(21)
    live = [synth.make_layer(s, l, 0) for l in range(2)]
    blobs = [synth.pack_blob(s, t) for t in live]
    dead = dict(live[0])
    for name in ("wo", "wd", "bo", "bd"):
        dead[name] = np.zeros_like(live[0][name])
    blob_dead = synth.pack_blob(s, dead)
    prompt = synth.to_bits(rng.standard_normal((B * P, s.hidden)), s.dtype)
    table = synth.to_bits(rng.standard_normal((2, B, s.hidden)), s.dtype)
    outs = {}
    for N in (0, 8):
        with Session(s, B, P + 4) as se:
            for l in range(L):
                sn.sn_set_layer_weights(se.ctx, l, blobs[l] if l < 2 else blob_dead)
            se.place(N)
            se.kv_reset([P + 4] * B)
            pre = se.step([P] * B, True, prompt)
            d0 = se.step([1] * B, False, table[0])
            d1 = se.step([1] * B, False, table[1])
            st = se.stats()
        assert st["n_offloaded"] == (L // N if N else 0)
        outs[N] = (pre, d0, d1)
    for a, b in zip(outs[0], outs[8]):
        assert np.array_equal(a, b)
        assert np.isfinite(synth.widen(a, s.dtype)).all()
    lws = [synth.widen_layer(s, t) for t in live]
    cache = ofw.new_cache(2, 1, s.n_kv_heads, s.head_dim)
    want = ofw.step(s.as_dict(), lws, [synth.widen(prompt[:40], s.dtype)], cache, kv_dtype=KV_STORAGE)[0]
    assert_close(outs[8][0][:40], want, s.dtype, "c2 full size, two live layers, sampled rows")


def _layer_rows(s, layer, x_seq, rows):
    """Oracle value of ONE layer's output for selected token rows of one sequence whose inputs to that layer are
    x_seq [P, hidden] (positions 0..P-1).  Keys and values are needed for every earlier position, everything else
    only for the selected rows, so the pieces of the oracle are applied to exactly those.  Both layer families."""
    Hq, Hkv, d, eps = s.n_q_heads, s.n_kv_heads, s.head_dim, s.norm_eps
    P = x_seq.shape[0]
    wd = lambda name: synth.widen(layer[name], s.dtype)
    norm = (lambda x, i: ofw.layer_norm(x, wd(f"n{i}g"), wd(f"n{i}b"), eps)) if s.norm == "ln" else \
           (lambda x, i: ofw.rms_norm(x, wd(f"n{i}g"), eps))
    bias = (lambda name: wd(name)) if s.has_bias else (lambda name: 0.0)
    u = norm(x_seq, 1)
    wqkv = wd("wqkv")
    bqkv = bias("bqkv")
    kv = u @ wqkv[Hq * d:].T + (bqkv[Hq * d:] if s.has_bias else 0.0)
    pos = np.arange(P)
    k = kv[:, :Hkv * d].reshape(P, Hkv, d)
    if s.rope:
        k = ofw.rope(k, pos[:, None], s.rope_theta)
    v = kv[:, Hkv * d:].reshape(P, Hkv, d)
    K, V = ofw.round_to_storage(k, KV_STORAGE), ofw.round_to_storage(v, KV_STORAGE)
    wq, wo, wdn = wqkv[:Hq * d], wd("wo"), wd("wd")
    wg = wd("wg") if s.act == "swiglu" else None
    wu = wd("wu")
    out = []
    for r in rows:
        q = (u[r] @ wq.T + (bqkv[:Hq * d] if s.has_bias else 0.0)).reshape(1, Hq, d)
        if s.rope:
            q = ofw.rope(q, np.array([[r]]), s.rope_theta)
        a = ofw.causal_attention(q, K[:r + 1], V[:r + 1], r).reshape(1, Hq * d)
        x1 = x_seq[r:r + 1] + a @ wo.T + bias("bo")
        u2 = norm(x1, 2)
        if s.act == "swiglu":
            m = ofw.silu(u2 @ wg.T + bias("bg")) * (u2 @ wu.T + bias("bu"))
        else:
            m = ofw.gelu(u2 @ wu.T + bias("bu"))
        out.append(x1 + m @ wdn.T + bias("bd"))
    return np.concatenate(out, axis=0)


def _two_live_layers_at_full_batch(name, P, rows_prompt, seed, **over):
    """A workload's real per-layer shape and full batch with 3 layers, the first two live and the third with its
    output projections zeroed (so the model IS its first two layers): offloaded runs -- interval 2; and interval 2
    with only the KV slices on the host under the continuous schedule -- are bit-identical to the all-resident one
    for the prefill and two decode steps, and the oracle reproduces sampled rows of sequence 0 through BOTH layers:
    layer 0 for every position of that sequence (layer 1's keys and values need them all), layer 1 for the sampled
    prompt positions and both decode steps."""
    import dataclasses
    w = synth.workload(name, **over)
    s = dataclasses.replace(w.shape, n_layers=3)
    B = w.batch
    lens = list(w.prompt_lens)          # ragged workloads: sequence 0 has P = lens[0] prompt tokens
    assert lens[0] == P and max(rows_prompt) < P
    T = sum(lens)
    rng = np.random.default_rng(seed)
    live = [synth.make_layer(s, l, 0) for l in range(2)]
    blobs = [synth.pack_blob(s, t) for t in live]
    dead = dict(live[0])
    for nm in ("wo", "wd") + (("bo", "bd") if s.has_bias else ()):
        dead[nm] = np.zeros_like(live[0][nm])
    blobs.append(synth.pack_blob(s, dead))
    del dead
    prompt = synth.to_bits(rng.standard_normal((T, s.hidden), dtype=np.float32), s.dtype)
    table = synth.to_bits(rng.standard_normal((2, B, s.hidden), dtype=np.float32), s.dtype)
    outs = {}
    for N in (0, 2, -2):            # -2: interval 2 again, KV slices only on the host, loads across the iteration boundary
        with Session(s, B, -(-(T + 4 * B) // B)) as se:
            for l in range(3):
                sn.sn_set_layer_weights(se.ctx, l, blobs[l])
            if N < 0:
                sn.sn_set_offload_part(se.ctx, sn.SN_OFFLOAD_KV)
                sn.sn_set_schedule(se.ctx, sn.SN_SCHED_CONTINUOUS)
            se.place(abs(N))
            se.kv_reset([p + 4 for p in lens])
            pre, fpre = se.step(lens, True, prompt, want_f32=True)
            d0, f0 = se.step([1] * B, False, table[0], want_f32=True)
            d1, f1 = se.step([1] * B, False, table[1], want_f32=True)
            st = se.stats()
        assert st["n_offloaded"] == (1 if N else 0)
        assert st["n_preissued"] == (1 if N < 0 else 0)
        outs[N] = (pre, d0, d1, fpre[:P].copy(), f0[0:1].copy(), f1[0:1].copy())
        del fpre
    for other in (2, -2):
        for a, b in zip(outs[0][:3], outs[other][:3]):
            assert np.array_equal(a, b)
    del blobs
    # oracle: sequence 0 = rows 0..P-1 of the prompt, then its two decode tokens at positions P, P+1
    x_seq = np.concatenate([synth.widen(prompt[:P], s.dtype), synth.widen(table[0, 0:1], s.dtype),
                            synth.widen(table[1, 0:1], s.dtype)], axis=0)
    y0 = ofw.layer_forward(s.as_dict(), synth.widen_layer(s, live[0]), x_seq,
                           {"k": np.zeros((0, s.n_kv_heads, s.head_dim)), "v": np.zeros((0, s.n_kv_heads, s.head_dim))},
                           KV_STORAGE)
    rows = list(rows_prompt) + [P, P + 1]
    want = _layer_rows(s, live[1], y0, rows)
    got_f = np.concatenate([outs[2][3][list(rows_prompt)], outs[2][4], outs[2][5]], axis=0)
    got_b = np.concatenate([outs[2][0][list(rows_prompt)], outs[2][1][0:1], outs[2][2][0:1]], axis=0)
    assert_close_f32(got_b, got_f, want, s.dtype, f"{name} shape, full batch, two live layers, sampled rows of sequence 0")


def test_full_size_config5_layer_shape_and_batch():
    """The Llama-2-70B-shaped configuration at its real per-layer shape and full batch: 64 sequences x 2048 prompt
    tokens = 131072 rows per prefill launch, GQA 64/8 heads, SwiGLU 28672, bf16 -- the launch configuration of that
    workload -- with 3 layers instead of 80 (the 80-layer model is 137 GB; the kernels do not depend on the layer
    count).  Sampled: early, tile-boundary and last prompt positions (attention over up to 2048 keys) and both
    decode steps (decode attention over 2049 / 2050 keys of layer 1's cache)."""
    _two_live_layers_at_full_batch("c5", 2048, [0, 1, 63, 64, 127, 128, 1023, 2047], 51)


def test_full_size_config4_layer_shape_ragged_batch_16():
    """The OPT-30B-shaped configuration at its real per-layer shape with its ragged prompts (256..2048 tokens, drawn as the
    benchmark draws them) at batch 16: LayerNorm, GELU, biases, 56 MHA heads x 128, FFN 28672; a prefill of ~15000 rows
    whose sequences end inside token tiles, and decode steps of 16 rows -- the one-row-tile instance of the LDS-sharing
    projection kernel and the split-K QKV projection summed by the attention kernel; 3 layers instead of 48."""
    P = synth.workload("c4", batch=16).prompt_lens[0]
    _two_live_layers_at_full_batch("c4", P, [0, 1, 15, 16, P // 2, P - 2, P - 1], 41, batch=16)


def test_full_size_config3_layer_shape_and_batch():
    """The Llama-2-13B-shaped configuration at its real per-layer shape, full batch and context: 32 sequences x 1024
    prompt tokens, 40 MHA heads (the vector decode-attention path, the largest kernel of that workload's decode
    step), SwiGLU 13824, bf16; 3 layers instead of 40."""
    _two_live_layers_at_full_batch("c3", 1024, [0, 1, 31, 32, 127, 128, 511, 1023], 31)
