"""The orderings the offloaded iteration depends on (paper Sec. 4.3, Fig. 7: the synchronisation
point before a host-resident layer; staging slots reused by later loads; state returning to the
host), forced instead of left to timing luck.  sn_set_debug poisons a staging slot as soon as it
is released and delays one of the three streams; with every combination the output has to stay
bit-identical to the all-resident run.  Iterations are enqueued back to back without any host
synchronisation in between, as a serving loop does.  Every added kernel ends by itself."""
import numpy as np
import pytest
import torch

from paper_2502_08182_amd import sn, synth
from paper_2502_08182_amd.runner import Session

pytestmark = pytest.mark.gpu

P, H, C, D = sn.SN_DEBUG_POISON_SLOT, sn.SN_DEBUG_DELAY_H2D, sn.SN_DEBUG_DELAY_COMPUTE, sn.SN_DEBUG_DELAY_D2H
# what each combination forces:
MODES = {
    "sync_point": P | H,      # compute arrives before the load has landed (the "S" of Fig. 7)
    "released_slot": P | C,   # the copy stream runs ahead: poison / the next layer land in a slot as soon as it is released
    "write_back": P | D,      # the KV slice a prefill produced reaches the host late
}
DELAY_US = 1000


def dev16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def run_back_to_back(se, w, prompt, table):
    """Prefill and all decode steps enqueued without waiting for the GPU in between."""
    with torch.cuda.stream(se.stream):
        x_pre = dev16(prompt)
        y_pre = torch.empty_like(x_pre)
        x_dec = [dev16(table[t]) for t in range(table.shape[0])]
        y_dec = [torch.empty_like(x) for x in x_dec]
    se.stream.synchronize()
    se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
    se.step_device(list(w.prompt_lens), True, x_pre, y_pre)
    for t in range(len(x_dec)):
        se.step_device([1] * w.batch, False, x_dec[t], y_dec[t])
    st = se.stats()                 # waits for the last iteration
    torch.cuda.synchronize()
    pre = y_pre.cpu().numpy().view(np.uint16)
    dec = np.stack([y.cpu().numpy().view(np.uint16) for y in y_dec]) if y_dec else np.zeros((0,), np.uint16)
    return pre, dec, st


@pytest.fixture(scope="module")
def c1():
    w = synth.workload("c1")
    layers = [synth.make_layer(w.shape, l, 0) for l in range(w.shape.n_layers)]
    prompt, table = synth.make_prompt(w), synth.make_decode_table(w)
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(0)
        pre, dec, _ = run_back_to_back(se, w, prompt, table)
    assert np.isfinite(synth.widen(pre, w.shape.dtype)).all() and np.isfinite(synth.widen(dec, w.shape.dtype)).all()
    return w, layers, prompt, table, pre, dec


@pytest.mark.parametrize("mode", sorted(MODES))
def test_forced_hazards_leave_the_output_bit_identical(c1, mode):
    w, layers, prompt, table, ref_pre, ref_dec = c1
    L = w.shape.n_layers
    for N in (1, 2):
        for sched in (sn.SN_SCHED_PAPER, sn.SN_SCHED_EAGER, sn.SN_SCHED_CONTINUOUS):
            for what in (sn.SN_OFFLOAD_STATE, sn.SN_OFFLOAD_WEIGHTS, sn.SN_OFFLOAD_KV):
                tag = f"mode={mode} N={N} schedule={sched} part={what}"
                print(tag, flush=True)
                with Session(w.shape, w.batch, w.max_seq) as se:
                    se.load_synthetic_weights(layers=layers)
                    sn.sn_set_offload_part(se.ctx, what)
                    sn.sn_set_schedule(se.ctx, sched)
                    se.place(N)
                    # baseline without switches: the second of two requests (the first one after a placement
                    # also pays for first-use effects of the pinned buffers and the copy engines)
                    run_back_to_back(se, w, prompt, table)
                    plain = run_back_to_back(se, w, prompt, table)[2]
                    sn.sn_set_debug(se.ctx, MODES[mode], DELAY_US)
                    pre, dec, st = run_back_to_back(se, w, prompt, table)
                    # twice: the second request starts while loads issued ahead for the first one's next step are around
                    pre2, dec2, _ = run_back_to_back(se, w, prompt, table)
                    sn.sn_set_debug(se.ctx, 0, 0)
                    pre3, dec3, _ = run_back_to_back(se, w, prompt, table)
                assert st["n_offloaded"] == L // N
                for a, b in ((pre, dec), (pre2, dec2), (pre3, dec3)):
                    assert np.array_equal(a, ref_pre), f"prefill differs: {tag}"
                    assert np.array_equal(b, ref_dec), f"decode differs: {tag}"
                if mode == "sync_point" and sched == sn.SN_SCHED_PAPER:
                    # every load of the last decode step started DELAY_US late and the layer that needs it could not
                    # run before it landed: the iteration is longer by about the delays.  (Usually all of it shows as
                    # waiting at the fence, stall_ns; but the runtime maps streams onto a few hardware queues, and when
                    # the copy stream shares one with the compute stream the delay holds up the kernels queued behind
                    # it instead -- so the check is on the iteration's length.)
                    assert st["iter_ns"] >= plain["iter_ns"] + 0.5 * DELAY_US * 1e3 * (L // N), \
                        (tag, st["iter_ns"], plain["iter_ns"], st["stall_ns"], plain["stall_ns"])


def test_debug_switch_rejects_bad_arguments(c1):
    w = c1[0]
    with Session(w.shape, w.batch, w.max_seq) as se:
        for flags, us in ((16, 0), (-1, 0), (1, -1), (2, 20001)):
            with pytest.raises(sn.SnError) as e:
                sn.sn_set_debug(se.ctx, flags, us)
            assert e.value.code == sn.SN_E_INVAL


def test_decode_right_after_a_prefill_whose_write_back_is_still_running():
    """One layer on the host (the case the picker returns most often), only its KV slice travelling, a slice of
    several hundred MB: the prefill's write-back of that slice takes milliseconds, the first decode step is
    enqueued at once.  Its load of the slice and the row its attention writes through must wait for the
    write-back (they use the other staging slot, so the slot's own release event does not order them)."""
    shape = synth.ModelShape(2, 1024, 8, 8, 128, 1024, act="gelu", norm="ln", rope=False, has_bias=True, dtype="f16")
    B, Pn, steps = 16, 4096, 3
    w = synth.Workload("kvbig", shape, B, (Pn,) * B, steps)
    layers = [synth.make_layer(shape, l, 0) for l in range(2)]
    prompt, table = synth.make_prompt(w), synth.make_decode_table(w)
    outs = {}
    for what, N in ((None, 0), (sn.SN_OFFLOAD_KV, 2), (sn.SN_OFFLOAD_STATE, 2)):
        with Session(shape, B, Pn + steps) as se:
            se.load_synthetic_weights(layers=layers)
            if what is not None:
                sn.sn_set_offload_part(se.ctx, what)
            se.place(N)
            pre, dec, st = run_back_to_back(se, w, prompt, table)
            assert st["n_offloaded"] == (1 if N else 0)
            if N:
                assert st["h2d_bytes"] >= B * Pn * shape.kv_bytes_per_token     # the slice travelled
        outs[what] = (pre, dec)
    assert np.isfinite(synth.widen(outs[None][1], "f16")).all()
    for what in (sn.SN_OFFLOAD_KV, sn.SN_OFFLOAD_STATE):
        assert np.array_equal(outs[what][0], outs[None][0]), what
        assert np.array_equal(outs[what][1], outs[None][1]), what


def test_kv_truncate_continues_from_the_shorter_cache(c1):
    """Dropping the newest rows and decoding again reproduces the steps that were dropped, bit for bit,
    under an offloading placement (the host slices keep the dropped rows until they are overwritten)."""
    w, layers, prompt, table, ref_pre, ref_dec = c1
    with Session(w.shape, w.batch, w.max_seq) as se:
        se.load_synthetic_weights(layers=layers)
        se.place(2)
        se.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        se.step(list(w.prompt_lens), True, prompt)
        first = [se.step([1] * w.batch, False, table[t]) for t in range(4)]
        with pytest.raises(sn.SnError) as e:
            sn.sn_kv_truncate(se.ctx, [p + 5 for p in w.prompt_lens])      # longer than what is cached
        assert e.value.code == sn.SN_E_INVAL
        se.kv_truncate([p + 1 for p in w.prompt_lens])
        se.place(1)
        again = [se.step([1] * w.batch, False, table[t]) for t in range(1, w.decode_steps)]
    assert np.array_equal(np.stack(first), ref_dec[:4])
    assert np.array_equal(np.stack(again), ref_dec[1:])
