#!/usr/bin/env python3
"""Benchmark of the offloaded serving iteration on one MI355X.

Default workload: the Llama-2-70B-shaped configuration, the largest one that fits one GPU (80 layers,
hidden 8192, 64 query / 8 KV heads, SwiGLU FFN 28672, bf16 random weights, 137 GB; batch 64, prompt
2048, teacher-forced decode), HBM budget 96 GB, TPOT SLO = 2 x the all-resident decode step.  One
"step" is one decode iteration of the whole layer loop (all kernels, prefetches, fences, write-through)
at the interval the picker chooses from the measured per-layer compute and transfer times.

Order of a run: weights -> profiles (whole state; KV slices only) -> ONE prefill -> all-resident decode
(defines TPOT and the SLO) -> pick -> decode at the picked interval (the headline) -> dominant kernel
timed inside iterations -> the same SLO under the continuous schedule and with only the KV slices on
the host -> CPU oracle.  The decode legs share the one prefill: the cache is cut back to the prompt
(sn_kv_truncate) and the placement changed (sn_place moves live state) between them.  --full adds
the looser SLO points, the interval sweep and the prefill phase with its own intervals.

Prints ONE JSON line (metric / value / roofline / cpu_baseline ...).  Inputs are resident in HBM
before the timed region.  Every timed iteration is synchronised and checked against the SLO, which is
how a serving loop consumes a decode step.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E
LINK_NOMINAL = 64.0e9      # bytes/s per direction, PCIe Gen5 x16 host link
MFMA_PEAK = 2.5e15         # flop/s, dense fp16/bf16 matrix cores
FAMILY = {"c2": "OPT-6.7B", "c3": "Llama-2-13B", "c4": "OPT-30B", "c5": "Llama-2-70B (GQA)"}
# rocprofv3 --pmc summaries of the dominant kernel (FETCH_SIZE / WRITE_SIZE), by (workload, batch)
TRAFFIC_NOTES = {("c2", 8): "gemm_skinny_ffn_up_c2_pmc.txt", ("c5", 64): "gemm_wide_ffn_up_c5_pmc.txt"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--slo-factor", type=float, default=None,
                    help="TPOT SLO as a multiple of the all-resident step (default: the workload's own, 2.0)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (the c4 batch sweep)")
    ap.add_argument("--guard", type=float, default=0.03,
                    help="fraction of the SLO kept as a guard band when picking (measured iterations run ~1-2%% "
                         "over the timeline's prediction: copies slow down slightly under concurrent compute)")
    ap.add_argument("--prefill-guard", type=float, default=0.06,
                    help="guard band of the prefill-phase picks: a prefill iteration keeps the link busy for most "
                         "of its length, where copies run 3-5%% slower than profiled in isolation")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB copy kernel (known HBM traffic) for counter calibration")
    ap.add_argument("--full", action="store_true",
                    help="also: the picker at looser SLOs, the interval sweep, the prefill phase with its own intervals, "
                         "weights-only offloading")
    ap.add_argument("--slo-points", default=None,
                    help="with --full: extra SLO factors (x all-resident TPOT) at which the picker is exercised and "
                         "verified (default: 3,5,10 for c2, the workload's other SLO factors otherwise)")
    ap.add_argument("--prefill-slo-points", default="1.2,1.5,2",
                    help="with --full: TTFT SLO factors (x all-resident prefill) at which the prefill phase picks its own interval")
    ap.add_argument("--host-limit-gb", type=float, default=24.0,
                    help="--full legs keep at most this much pinned host memory: sweep points beyond it are skipped, "
                         "prefill picks are moved to the first interval within it")
    ap.add_argument("--contention", type=float, default=0.0, metavar="FRACTION",
                    help="also run the prefill phase while a competing host-to-device copy stream takes this fraction "
                         "of the link (0: off): at the interval picked without contention, then at the interval the "
                         "bandwidth coordinator assigns (Sec. 4.5)")
    ap.add_argument("--repick", type=int, default=0, metavar="CELLS",
                    help="also run the decode steps with the interval re-selected before every iteration from a "
                         "performance record of CELLS sequence lengths spanning the run (the KV cache grows, the "
                         "TPOT SLO stays fixed); 0: off")
    ap.add_argument("--no-continuous", action="store_true",
                    help="skip the decode run with loads issued across the iteration boundary")
    ap.add_argument("--no-parts", action="store_true",
                    help="skip the decode runs with only the KV slices of host-resident layers on the host")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--distinct-layers", type=int, default=0,
                    help="draw only this many different random layer blobs (0: every layer its own)")
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic_note(name):
    """HBM bytes per launch measured offline with rocprofv3 --pmc (profiles/<name>), or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


class DecodeRig:
    """One prefill, then any number of decode legs over the same prompt cache: a leg cuts the cache back to
    the prompt (sn_kv_truncate), runs warm-up steps and then timed steps, each synchronised."""

    def __init__(self, se, sn, torch, w, x_pre, y_pre, x_dec, y_dec, max_steps):
        self.se, self.sn, self.torch, self.w = se, sn, torch, w
        self.x_pre, self.y_pre, self.x_dec, self.y_dec = x_pre, y_pre, x_dec, y_dec
        self.max_steps = max_steps
        self.prefilled = False

    def prefill(self):
        se, sn, w = self.se, self.sn, self.w
        se.kv_reset([p + self.max_steps + 1 for p in w.prompt_lens])
        sn.sn_set_timing(se.ctx, 0)
        se.step_device(list(w.prompt_lens), True, self.x_pre, self.y_pre)
        self.prefilled = True
        return sn.sn_get_stats(se.ctx).as_dict()

    def decode(self, n_steps, warmup, timing_class=None):
        """Returns per-step stats and wall ms per step of n_steps timed decode iterations."""
        se, sn, torch, w = self.se, self.sn, self.torch, self.w
        assert warmup + n_steps <= self.max_steps
        if not self.prefilled:
            self.prefill()
        se.kv_truncate(list(w.prompt_lens))
        sn.sn_set_timing(se.ctx, 0)
        ones = [1] * w.batch
        for i in range(warmup):
            se.step_device(ones, False, self.x_dec[i % len(self.x_dec)], self.y_dec)
        se.stream.synchronize()
        if timing_class is not None:
            sn.sn_set_timing(se.ctx, 2)
            sn.sn_set_kernel_timing_class(se.ctx, timing_class)
        stats = []
        torch.cuda.synchronize()
        gc_was_on = gc.isenabled()
        gc.disable()                                       # no collector pauses inside the timed region
        t0 = time.perf_counter()
        for i in range(n_steps):
            se.step_device(ones, False, self.x_dec[i % len(self.x_dec)], self.y_dec)
            stats.append(sn.sn_get_stats(se.ctx))          # synchronises the iteration
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / n_steps
        if gc_was_on:
            gc.enable()
        sn.sn_set_timing(se.ctx, 0)
        sn.sn_set_kernel_timing_class(se.ctx, -1)
        return [s.as_dict() for s in stats], wall_ms


def leg_summary(stats, wall_ms, slo_ns, B):
    it = np.array([d["iter_ns"] for d in stats], dtype=np.float64)
    h = sum(d["h2d_ns"] for d in stats)
    hb = sum(d["h2d_bytes"] for d in stats)
    st = sum(d["stall_ns"] for d in stats)
    return {"n_offloaded": int(stats[-1]["n_offloaded"]), "tpot_median_ms": float(np.median(it)) / 1e6,
            "tpot_max_ms": float(it.max()) / 1e6, "every_iteration_within_slo": bool((it <= slo_ns).all()),
            "hidden_fraction": (1.0 - st / h) if h else 1.0, "h2d_GBps": (hb / (h * 1e-9) / 1e9) if h else None,
            "h2d_bytes_per_step": hb / len(stats), "stall_ms_per_step": st / len(stats) / 1e6,
            "tokens_per_s": B * 1e3 / wall_ms, "tokens_per_s_at_median_tpot": B / (float(np.median(it)) * 1e-9)}


def run_prefill(se, sn, w, x_pre, y_pre, reps=2):
    """reps prefill iterations from empty caches, each synchronised; returns their stats."""
    out = []
    sn.sn_set_timing(se.ctx, 0)
    for _ in range(reps):
        se.kv_reset([p + 1 for p in w.prompt_lens])
        se.step_device(list(w.prompt_lens), True, x_pre, y_pre)
        out.append(sn.sn_get_stats(se.ctx).as_dict())
    return out


def cpu_baseline(w, seconds_target=12.0):
    """The CPU oracle on decode steps at the real shape: a bounded sample of about 10-20 s.  One step is
    n_layers passes of oracle.forward.layer_forward over the whole batch; all passes use layer 0's
    weights (float64 copies of every layer would need tens of GB) -- the arithmetic is the same."""
    from oracle import forward as ofw
    from paper_2502_08182_amd import synth
    s = w.shape
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    layer = synth.widen_layer(s, synth.make_layer(s, 0, 0))
    rng = np.random.default_rng(7)
    B, P = w.batch, int(round(float(np.mean(w.prompt_lens))))
    kv = [{"k": ofw.round_to_storage(rng.standard_normal((P, s.n_kv_heads, s.head_dim)), s.dtype),
           "v": ofw.round_to_storage(rng.standard_normal((P, s.n_kv_heads, s.head_dim)), s.dtype)} for _ in range(B)]
    x = rng.standard_normal((B, s.hidden))
    sd = s.as_dict()
    step_times, layer_passes = [], 0
    t_all = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        partial = False
        for _ in range(s.n_layers):
            caches = [dict(c) for c in kv]
            for b in range(B):
                ofw.layer_forward(sd, layer, x[b:b + 1], caches[b])
            layer_passes += 1
            if not step_times and time.perf_counter() - t_all > 2.5 * seconds_target:
                partial = True            # a step would take minutes (the 70B shape): keep what was measured
                break
        dt = time.perf_counter() - t0
        if partial:
            step_times.append(dt * s.n_layers / layer_passes)
            break
        step_times.append(dt)
        if time.perf_counter() - t_all > seconds_target or len(step_times) >= 6:
            break
    t_step = float(np.median(step_times))
    total = time.perf_counter() - t_all
    return {"value": B / t_step, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{layer_passes} layer passes of the float64 numpy oracle at the real shape (batch {B}, {P} cached "
                      f"tokens per sequence) in {total:.1f} s; a decode step = {s.n_layers} passes = {t_step * 1e3:.0f} ms "
                      f"(median of {len(step_times)} step{'s' if len(step_times) != 1 else ''}"
                      f"{', scaled from a partial step' if layer_passes < s.n_layers else ''}); every pass uses layer 0's weights"}


def pick_or_none(sn, tc, tx, slo_ns, n_max, sched):
    """Smallest interval meeting slo_ns under `sched`, L + 1 when only the un-offloaded iteration does."""
    try:
        return sn.sn_pick_interval_from_times_sched(tc, tx, int(slo_ns), n_max, sched)
    except sn.SnError as e:
        if e.code != sn.SN_E_INFEASIBLE:
            raise
        return len(tc) + 1


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one model instance per GPU, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2502_08182_amd import sn, synth
    from paper_2502_08182_amd.runner import Session

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    w = synth.workload(a.workload, **({"batch": a.batch} if a.batch and a.workload == "c4" else {}))
    if a.batch and a.workload != "c4":
        from dataclasses import replace
        w = replace(w, batch=a.batch, prompt_lens=(w.prompt_lens[0],) * a.batch)
    s = w.shape
    L, B = s.n_layers, w.batch
    K, W = a.steps, a.warmup
    if a.slo_factor is None:
        a.slo_factor = max(w.slo_factors) if w.slo_factors else 2.0
    if a.slo_points is None:
        a.slo_points = "3,5,10" if w.name == "c2" else ",".join(str(f) for f in w.slo_factors if f != a.slo_factor)
    p_mean = int(round(float(np.mean(w.prompt_lens))))      # ragged prompts: profile at the mean length
    # KV capacity: the context holds max_batch * max_seq tokens per layer in all; ragged prompts need their sum, not B x the longest
    max_seq = -(-sum(p + K + W + 2 for p in w.prompt_lens) // B)
    t_start = time.time()
    se = Session(s, B, max_seq, hbm_budget=w.hbm_budget)
    sn.sn_set_budget_enforce(se.ctx, False)     # over-cap intervals are run and labelled, not refused
    log(f"[bench] {w.name}: L={L} h={s.hidden} heads={s.n_q_heads}/{s.n_kv_heads} ffn={s.ffn} {s.dtype} "
        f"B={B} P={min(w.prompt_lens)}..{max(w.prompt_lens)} (mean {p_mean}) budget={w.hbm_budget / 1e9:.1f} GB")
    se.place(0)       # weights go straight to the device; host masters only for layers that get offloaded
    se.load_device_generated_weights(seed=0, distinct=a.distinct_layers)
    log(f"[bench] weights loaded in {time.time() - t_start:.1f} s")

    tdt = torch.bfloat16 if s.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    T = int(sum(w.prompt_lens))
    with torch.cuda.stream(se.stream):
        x_pre = torch.empty(T, s.hidden, device="cuda", dtype=tdt)
        for r0 in range(0, T, 8192):                           # in pieces: no fp32 copy of the whole prompt
            r1 = min(T, r0 + 8192)
            x_pre[r0:r1] = torch.randn(r1 - r0, s.hidden, generator=g, device="cuda", dtype=torch.float32).to(tdt)
        y_pre = torch.empty_like(x_pre)
        g.manual_seed(2)
        x_dec = [torch.randn(B, s.hidden, generator=g, device="cuda", dtype=torch.float32).to(tdt) for _ in range(8)]
        y_dec = torch.empty_like(x_dec[0])
    se.stream.synchronize()

    kvtok = s.kv_bytes_per_token
    w_layer = sn.sn_layer_blob_bytes(se.cshape)
    seq_prof = p_mean + W + K // 2               # the decode legs' mid-run cache length
    PAPER, CONT = sn.SN_SCHED_PAPER, sn.SN_SCHED_CONTINUOUS

    # ---- profiles (Sec. 4.4), before the prefill: the profiler runs on generated inputs and leaves the caches empty
    t_prof = time.time()
    profiles = {}
    parts_wanted = ([] if a.no_parts else ["kv"]) + (["weights"] if a.full and not a.no_parts else [])
    for name in parts_wanted:
        sn.sn_set_offload_part(se.ctx, sn.SN_OFFLOAD_KV if name == "kv" else sn.SN_OFFLOAD_WEIGHTS)
        profiles[name] = sn.sn_profile_layers(se.ctx, L, False, B, seq_prof, reps=3)
    sn.sn_set_offload_part(se.ctx, sn.SN_OFFLOAD_STATE)
    tc, tx = sn.sn_profile_layers(se.ctx, L, False, B, seq_prof, reps=3)     # last: the one sn_pick_interval uses
    profiles["state"] = (tc, tx)
    rho = float(np.median(tx) / np.median(tc))
    log(f"[bench] profiles ({', '.join(profiles)}) in {time.time() - t_prof:.1f} s: tc median {np.median(tc) / 1e3:.1f} us, "
        f"tx median {np.median(tx) / 1e3:.1f} us, rho {rho:.1f}, cv(tc) {np.std(tc) / np.mean(tc):.4f}")

    # ---- ONE prefill, then the all-resident reference: defines the SLO (TPOT without offloading) -----
    rig = DecodeRig(se, sn, torch, w, x_pre, y_pre, x_dec, y_dec, K + W)
    pre0 = rig.prefill()
    rig.decode(min(K, 8), W)                                  # untimed pass: clocks and caches settle
    st0, wall0 = rig.decode(K, W)
    it0 = np.array([d["iter_ns"] for d in st0], dtype=np.float64)
    tpot0_ns = float(np.median(it0))
    slo_ns = int(a.slo_factor * tpot0_ns)
    log(f"[bench] all-resident: TPOT median {tpot0_ns / 1e6:.3f} ms (max {it0.max() / 1e6:.3f}), wall {wall0:.3f} ms/step, "
        f"prefill {pre0['iter_ns'] / 1e6:.2f} ms; SLO = {a.slo_factor} x = {slo_ns / 1e6:.3f} ms")

    # ---- where the all-resident decode step spends its time: each projection class timed alone, back to back
    # over every layer's own weights (one pair of HIP events around the region); attention, the norms and the
    # casts are what remains of the layer time ----
    n_up = s.ffn * (2 if s.act == "swiglu" else 1)
    qd0 = s.n_q_heads * s.head_dim
    class_bytes = {"qkv": (qd0 + 2 * s.n_kv_heads * s.head_dim) * s.hidden * 2, "oproj": s.hidden * qd0 * 2,
                   "ffn_up": n_up * s.hidden * 2, "ffn_down": s.hidden * s.ffn * 2}
    breakdown = {}
    for name, cls in (("qkv", 1), ("oproj", 4), ("ffn_up", 5), ("ffn_down", 6)):
        ns, calls = sn.sn_time_kernel_class(se.ctx, cls, B, reps=2)
        us = ns / max(calls, 1) / 1e3
        gbps = class_bytes[name] / (us * 1e-6) / 1e9
        breakdown[name] = {"us_per_launch": us, "weight_MB": class_bytes[name] / 1e6, "GBps": gbps, "frac_of_hbm_peak": gbps * 1e9 / HBM_PEAK}
    layer_us = tpot0_ns / L / 1e3
    rest_us = layer_us - sum(v["us_per_launch"] for v in breakdown.values())
    kv_mb = seq_prof * B * kvtok / 1e6
    breakdown["attention_norms_casts"] = {"us_per_layer": rest_us, "kv_MB_per_layer": kv_mb}
    breakdown["layer_us"] = layer_us
    log("[bench] decode layer %.1f us: " % layer_us + ", ".join(
        f"{k} {v['us_per_launch']:.1f} us ({v['GBps'] / 1e3:.2f} TB/s)" for k, v in breakdown.items() if isinstance(v, dict) and "GBps" in v)
        + f", attention + norms + casts {rest_us:.1f} us (KV {kv_mb:.0f} MB)")

    # ---- pick (Sec. 4.3 / 4.4) and the admission check against the capacity bound (Sec. 4.5) -------------
    n_max_cap = sn.sn_max_interval(se.ctx)
    pick_slo_ns = int(slo_ns * (1.0 - a.guard))
    n_min = pick_or_none(sn, tc, tx, pick_slo_ns, L + 1, PAPER)
    try:
        n_pick_cap = sn.sn_pick_interval(se.ctx, pick_slo_ns / 1e6)      # the last profile, the budget, the schedule
        feasible_at_cap = True
    except sn.SnError as e:
        if e.code != sn.SN_E_INFEASIBLE:
            raise
        n_pick_cap, feasible_at_cap = None, False
    pred_ns, _ = sn.sn_timeline(tc, tx, n_min)
    n_paper = sn.sn_paper_rule(L, int(np.median(tx)), slo_ns)
    log(f"[bench] N_min(SLO)={n_min} N_max(cap)={n_max_cap} feasible_at_cap={feasible_at_cap} paper_rule={n_paper} "
        f"predicted T(N_min)={pred_ns / 1e6:.3f} ms")
    n_first = n_pick_cap if feasible_at_cap else n_min
    # intervals that offload as many layers as the smallest one that meets the SLO hold the same host memory; of
    # those, the one with the shortest predicted iteration runs (sn_refine_interval_from_times)
    n_run = sn.sn_refine_interval_from_times(tc, tx, n_first, PAPER)
    smallest_leg = None
    if n_run != n_first:
        se.place(n_first)
        st1, wall1 = rig.decode(min(K, 16), W)
        smallest_leg = {"interval": int(n_first), **leg_summary(st1, wall1, slo_ns, B),
                        "predicted_ms": sn.sn_timeline(tc, tx, n_first)[0] / 1e6}
        log(f"[bench] smallest interval meeting the SLO N={n_first} (K={smallest_leg['n_offloaded']}): TPOT median "
            f"{smallest_leg['tpot_median_ms']:.3f} ms max {smallest_leg['tpot_max_ms']:.3f} ms -> {smallest_leg['tokens_per_s']:.1f} tok/s, "
            f"hidden {smallest_leg['hidden_fraction']:.3f}; same host memory at N={n_run}: predicted "
            f"{sn.sn_timeline(tc, tx, n_run)[0] / 1e6:.3f} ms")

    # ---- the measured run at the picked interval: the headline ---------------------------------------------
    se.place(n_run)
    st, wall_ms = rig.decode(K, W)
    head = leg_summary(st, wall_ms, slo_ns, B)
    pred_ns, _ = sn.sn_timeline(tc, tx, n_run)
    it = np.array([d["iter_ns"] for d in st], dtype=np.float64)
    value = B * 1e3 / wall_ms
    log(f"[bench] N={n_run} (K={head['n_offloaded']}): TPOT median {head['tpot_median_ms']:.3f} ms max {head['tpot_max_ms']:.3f} ms "
        f"(SLO {slo_ns / 1e6:.3f}), wall {wall_ms:.3f} ms/step -> {value:.1f} tok/s, hidden {head['hidden_fraction']:.3f}")

    # ---- the dominant kernel (FFN up-projection of the decode step), timed live: (i) inside iterations under this
    # placement, each launch bracketed by its own start/stop timestamps (what a kernel trace shows); (ii) on its own,
    # back to back over every resident layer's weights between one pair of events (launch gaps included) ----------
    kst, _ = rig.decode(min(K, 4), 1, timing_class=5)
    in_ns = sum(d["kernel_ns"]["ffn_up"] for d in kst)
    in_calls = sum(d["kernel_calls"]["ffn_up"] for d in kst)
    k_ns, k_calls = sn.sn_time_kernel_class(se.ctx, 5, B, reps=4)
    # algorithmic bytes per launch: weights + bias + activations in + out
    alg_bytes = n_up * s.hidden * 2 + (n_up * 2 if s.has_bias else 0) + B * s.hidden * 2 + B * s.ffn * 2
    in_avg_ns = in_ns / max(in_calls, 1)
    k_avg_ns = k_ns / max(k_calls, 1)
    achieved = alg_bytes / (k_avg_ns * 1e-9) if k_avg_ns > 0 else 0.0
    note = TRAFFIC_NOTES.get((w.name, B))
    traffic = read_traffic_note(note) if note else None
    roofline = {"bound": "hbm", "kernel": "FFN up-projection of the decode step (gemm_wide_kernel / gemm_skinny_kernel)", "achieved": achieved / 1e9,
                "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": achieved / HBM_PEAK, "traffic": traffic,
                "traffic_source": (f"profiles/{note}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, collected offline "
                                   "(hardware counters cannot be read from inside the run)") if traffic else None,
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": k_avg_ns / 1e3, "launches_timed": k_calls,
                "timed": "one pair of HIP events on the compute stream around back-to-back launches on every resident layer's own weights "
                         "(launch gaps included); agrees with the kernel trace's average inside iterations",
                "inside_iterations": {"avg_launch_us": in_avg_ns / 1e3, "launches": in_calls,
                                      "GBps": alg_bytes / (in_avg_ns * 1e-9) / 1e9 if in_avg_ns > 0 else None,
                                      "note": "each launch bracketed by its own start/stop events, which add a few microseconds"}}
    log(f"[bench] ffn_up back to back {k_avg_ns / 1e3:.1f} us = {achieved / 1e9:.0f} GB/s ({k_calls} launches); "
        f"inside iterations, bracketed {in_avg_ns / 1e3:.1f} us")
    # whole-step HBM roofline: every weight and every cached K/V element is read once per step
    step_bytes = L * (w_layer + seq_prof * B * kvtok)
    # prefill: dense contractions.  2 flop per weight element per token, plus causal attention
    # (QK^T and PV: 4 * Hq * d flop per (query, visible key) pair)
    w_elems = s.hidden * (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim + s.n_q_heads * s.head_dim * s.hidden \
        + s.hidden * s.ffn * (3 if s.act == "swiglu" else 2)
    pre_flops = L * (2.0 * w_elems * T + 4.0 * s.n_q_heads * s.head_dim * sum(p * (p + 1) / 2 for p in w.prompt_lens))
    over_cap = bool(sn.sn_resident_bytes(se.ctx, n_run) > w.hbm_budget > 0)

    out = {
        "metric": "decode tok/s at max-offload interval meeting TPOT SLO; HBM + H2D GB/s",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16" if s.dtype == "f16" else "f16 (bf16 storage)",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {FAMILY.get(w.name, w.name)}-shaped decoder, {L} layers, hidden {s.hidden}, "
                               f"{s.n_q_heads} query / {s.n_kv_heads} KV heads, {'SwiGLU' if s.act == 'swiglu' else 'GELU'} FFN "
                               f"{s.ffn}, {'fp16' if s.dtype == 'f16' else 'bf16'} random weights N(0,0.02), batch {B}, prompt "
                               f"{w.prompt_lens[0] if min(w.prompt_lens) == max(w.prompt_lens) else f'{min(w.prompt_lens)}..{max(w.prompt_lens)}'}"
                               f", teacher-forced decode; HBM budget {w.hbm_budget / 1e9:.0f} GB; TPOT SLO {a.slo_factor}x all-resident",
                   "interval": int(n_run), "n_offloaded": head["n_offloaded"], "schedule": "paper (Fig. 7)",
                   "interval_smallest_meeting_slo": int(n_first),
                   "interval_rule": "smallest interval that meets the SLO (Sec. 4.3 / 4.4: the most layers on the host), then, of the "
                                    "intervals that offload as many layers (same host memory), the one with the shortest predicted iteration",
                   "host_resident_GB": head["n_offloaded"] * (w_layer + seq_prof * B * kvtok) / 1e9,
                   "interval_over_cap": over_cap,
                   "admission_at_cap": ("feasible" if feasible_at_cap else
                                        f"SN_E_INFEASIBLE: smallest interval meeting the SLO is {n_min}, largest the {w.hbm_budget / 1e9:.0f} GB "
                                        f"cap holds is {n_max_cap}; under Sec. 4.5 this request goes back to the scheduler.  Timed with the "
                                        f"cap lifted (the device holds 288 GB) at the interval `interval_rule` gives")},
        "roofline": roofline,
        "slo": {"tpot_all_resident_ms": tpot0_ns / 1e6, "slo_ms": slo_ns / 1e6, "tpot_median_ms": head["tpot_median_ms"],
                "tpot_max_ms": head["tpot_max_ms"], "every_iteration_within_slo": head["every_iteration_within_slo"],
                "guard_band": a.guard, "n_min_slo": int(n_min), "n_max_cap": int(n_max_cap), "feasible_at_cap": feasible_at_cap,
                "paper_closed_form_interval": int(n_paper), "predicted_iter_ms": pred_ns / 1e6,
                "rho_transfer_over_compute": rho, "layer_compute_us_median": float(np.median(tc)) / 1e3,
                "layer_transfer_us_median": float(np.median(tx)) / 1e3,
                "layer_compute_cv": float(np.std(tc) / np.mean(tc))},
        "h2d": {"bytes_per_step": head["h2d_bytes_per_step"], "achieved_GBps": head["h2d_GBps"],
                "solo_GBps": float((w_layer + seq_prof * B * kvtok) / (np.median(tx) * 1e-9) / 1e9),
                "nominal_link_GBps": LINK_NOMINAL / 1e9,
                "hidden_fraction": head["hidden_fraction"], "stall_ms_per_step": head["stall_ms_per_step"]},
        "hbm_step": {"algorithmic_bytes_per_step": step_bytes, "all_resident_GBps": step_bytes / (tpot0_ns * 1e-9) / 1e9,
                     "frac_of_peak": step_bytes / (tpot0_ns * 1e-9) / HBM_PEAK,
                     "all_resident_tokens_per_s": B / (tpot0_ns * 1e-9),
                     "roofline_tokens_per_s": B * HBM_PEAK / step_bytes},
        "decode_at_smallest_interval_meeting_slo": smallest_leg,
        "decode_layer_breakdown": breakdown,
        "prefill": {"iter_ms_all_resident": pre0["iter_ns"] / 1e6, "tokens": T, "algorithmic_tflop": pre_flops / 1e12,
                    "all_resident_TFLOPs": pre_flops / (pre0["iter_ns"] * 1e-9) / 1e12,
                    "frac_of_mfma_peak": pre_flops / (pre0["iter_ns"] * 1e-9) / MFMA_PEAK},
    }

    # Sec. 5.6 / Fig. 14: tokens ("max length" = batch x (sequence + output)) the HBM budget can hold per interval
    if w.hbm_budget > 0:
        base_tok = sn.sn_max_tokens(L, 0, w_layer, kvtok, 0, w.hbm_budget)
        out["max_length_vs_interval"] = {
            "hbm_budget_GB": w.hbm_budget / 1e9, "workspace": "excluded",
            "rows": [{"interval": int(N), "max_tokens": int(sn.sn_max_tokens(L, N, w_layer, kvtok, 0, w.hbm_budget)),
                      "max_tokens_weights_only": int(sn.sn_max_tokens_part(L, N, w_layer, kvtok, 0, w.hbm_budget, sn.SN_OFFLOAD_WEIGHTS)),
                      "max_tokens_kv_only": int(sn.sn_max_tokens_part(L, N, w_layer, kvtok, 0, w.hbm_budget, sn.SN_OFFLOAD_KV))}
                     for N in sorted({1, 2, 3, 4, 6, 8, 16, L, L + 1}) if N <= L + 1],
            "no_offloading_tokens": int(base_tok)}

    if a.calibrate_copy:
        from paper_2502_08182_amd import sn_kernels
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        sn_kernels.sn_k_copy(src, dst, 1 << 30, se.stream.cuda_stream)
        se.stream.synchronize()
        del src, dst

    def decode_point(f, tcp_, txp_, sched, steps):
        """Pick for SLO f x the all-resident TPOT under `sched` from the given profile, place, run, check."""
        slo_f = int(f * tpot0_ns)
        n_f = pick_or_none(sn, tcp_, txp_, int(slo_f * (1.0 - a.guard)), L + 1, sched)
        smallest = int(n_f)
        n_f = sn.sn_refine_interval_from_times(tcp_, txp_, n_f, sched)     # same layers on the host, shortest iteration
        first = int(n_f)
        # an interval whose measured iterations miss the SLO (the analyzer's prediction leaves out what many small
        # copies and the fences cost) is replaced by the next one that offloads fewer layers, and run again
        for _ in range(4):
            se.place(n_f)
            fst, fwall = rig.decode(steps, W)
            k_f = int(fst[-1]["n_offloaded"])
            if k_f == 0 or all(d["iter_ns"] <= slo_f for d in fst):
                break
            n_next = n_f + 1
            while n_next <= L and L // n_next >= k_f:
                n_next += 1
            log(f"[bench] SLO {f}x: N={n_f} measured {max(d['iter_ns'] for d in fst) / 1e6:.3f} ms > SLO {slo_f / 1e6:.3f}, trying N={n_next}"
                + " (iterations, ms: " + " ".join("%.2f" % (d["iter_ns"] / 1e6) for d in fst)
                + "; stalls, ms: " + " ".join("%.2f" % (d["stall_ns"] / 1e6) for d in fst) + ")")
            n_f = n_next
        pt = {"slo_factor": f, "slo_ms": slo_f / 1e6, "picked_interval": int(n_f), "smallest_interval_meeting_slo": smallest,
              "picker_first_choice": first,
              "adjusted_after_measurement": bool(first != int(n_f)), **leg_summary(fst, fwall, slo_f, B)}
        pred, _ = sn.sn_timeline_sched(tcp_, txp_, n_f, sched)
        pt["predicted_ms"] = pred / 1e6
        pt["resident_GB"] = sn.sn_resident_bytes(se.ctx, n_f) / 1e9
        pt["over_cap"] = bool(sn.sn_resident_bytes(se.ctx, n_f) > w.hbm_budget > 0)
        pt["loads_issued_ahead_per_step"] = int(fst[-1]["n_preissued"])
        return pt

    k_short = min(K, 16)
    extra_factors = [float(v) for v in a.slo_points.split(",") if v] if (a.full and a.slo_points) else []

    # ---- the picker at looser SLOs: pick, run, check every iteration (over-cap points labelled) ----
    if extra_factors:
        pts = []
        for f in extra_factors:
            pts.append(decode_point(f, tc, tx, PAPER, min(K, 8)))
            log(f"[bench] SLO {f}x: picked N={pts[-1]['picked_interval']} (K={pts[-1]['n_offloaded']}), TPOT median "
                f"{pts[-1]['tpot_median_ms']:.3f} max {pts[-1]['tpot_max_ms']:.3f} (predicted {pts[-1]['predicted_ms']:.3f}) "
                f"within={pts[-1]['every_iteration_within_slo']} hidden {pts[-1]['hidden_fraction']:.3f}")
        out["slo_points"] = pts

    # ---- decode with loads that run on across the iteration boundary (continuous schedule): the steady
    # state the analyzer's closed form describes -- floor(SLO / transfer) layers fit one iteration -----------
    if not a.no_continuous:
        sn.sn_set_schedule(se.ctx, CONT)
        cont = []
        for f in [a.slo_factor] + extra_factors:
            pt = decode_point(f, tc, tx, CONT, k_short)
            pt["interval_picked_for_the_papers_schedule"] = int(pick_or_none(sn, tc, tx, int(f * tpot0_ns * (1.0 - a.guard)), L + 1, PAPER))
            pt["predicted_papers_schedule_ms"] = sn.sn_timeline(tc, tx, pt["picked_interval"])[0] / 1e6
            pt["host_resident_GB"] = pt["n_offloaded"] * (w_layer + seq_prof * B * kvtok) / 1e9
            cont.append(pt)
            log(f"[bench] continuous schedule, SLO {f}x: picked N={pt['picked_interval']} (K={pt['n_offloaded']}), TPOT median "
                f"{pt['tpot_median_ms']:.3f} max {pt['tpot_max_ms']:.3f} (predicted {pt['predicted_ms']:.3f}; paper's schedule at this N "
                f"{pt['predicted_papers_schedule_ms']:.3f}) within={pt['every_iteration_within_slo']} hidden {pt['hidden_fraction']:.3f} "
                f"issued ahead {pt['loads_issued_ahead_per_step']} -> {pt['tokens_per_s']:.1f} tok/s")
        sn.sn_set_schedule(se.ctx, PAPER)
        out["decode_continuous_schedule"] = cont

    # ---- host-resident layers that keep only their KV slice (or only their weights) on the host: smaller
    # loads, so the same SLO admits more layers (at the price of the part that stays on the GPU) ---------------
    if parts_wanted:
        parts = []
        for name in parts_wanted:
            what = sn.SN_OFFLOAD_KV if name == "kv" else sn.SN_OFFLOAD_WEIGHTS
            tcw, txw = profiles[name]
            se.place(0)
            sn.sn_set_offload_part(se.ctx, what)
            row = {"part_on_host": name, "layer_transfer_us_median": float(np.median(txw)) / 1e3,
                   "rho_transfer_over_compute": float(np.median(txw) / np.median(tcw)), "points": []}
            for sched, sname in ((PAPER, "paper"), (CONT, "continuous")):
                sn.sn_set_schedule(se.ctx, sched)
                pt = decode_point(a.slo_factor, tcw, txw, sched, k_short)
                pt["schedule"] = sname
                pt["host_resident_GB"] = pt["n_offloaded"] * (w_layer if name == "weights" else seq_prof * B * kvtok) / 1e9
                row["points"].append(pt)
                log(f"[bench] {name} only on the host, {sname} schedule, SLO {a.slo_factor}x: tx {row['layer_transfer_us_median']:.0f} us "
                    f"(rho {row['rho_transfer_over_compute']:.1f}); picked N={pt['picked_interval']} (K={pt['n_offloaded']}, "
                    f"{pt['host_resident_GB']:.2f} GB on the host), TPOT median {pt['tpot_median_ms']:.3f} max {pt['tpot_max_ms']:.3f} "
                    f"(predicted {pt['predicted_ms']:.3f}) within={pt['every_iteration_within_slo']} hidden {pt['hidden_fraction']:.3f}")
            sn.sn_set_schedule(se.ctx, PAPER)
            parts.append(row)
        se.place(0)
        sn.sn_set_offload_part(se.ctx, sn.SN_OFFLOAD_STATE)
        out["decode_by_offloaded_part"] = parts

    # ---- interval sweep (reported, over-cap points labelled) ------------------------------------
    if a.full:
        sweep = []
        state_bytes = w_layer + seq_prof * B * kvtok
        for N in list(w.intervals) + [L]:
            if (L // N) * state_bytes > a.host_limit_gb * 1e9:
                log(f"[bench] sweep N={N}: skipped, {(L // N) * state_bytes / 1e9:.0f} GB of pinned host memory (--host-limit-gb)")
                continue
            log(f"[bench] sweep N={N}: placing {L // N} layers on the host")
            se.place(N)
            sst, swall = rig.decode(min(K, 8), 1)
            row = {"interval": N, **leg_summary(sst, swall, slo_ns, B)}
            pred, _ = sn.sn_timeline(tc, tx, N)
            row.update({"x_all_resident": row["tpot_median_ms"] * 1e6 / tpot0_ns, "predicted_ms": pred / 1e6,
                        "resident_GB": sn.sn_resident_bytes(se.ctx, N) / 1e9,
                        "over_cap": bool(sn.sn_resident_bytes(se.ctx, N) > w.hbm_budget > 0)})
            sweep.append(row)
            log(f"[bench] sweep N={N}: TPOT {row['tpot_median_ms']:.3f} ms ({row['x_all_resident']:.2f}x, predicted "
                f"{pred / 1e6:.3f}) hidden {row['hidden_fraction']:.3f} h2d {row['h2d_GBps']} GB/s")
        out["sweep"] = sweep
    se.place(0)

    # ---- the prefill phase has its own profile and its own interval (Sec. 4.4, separation of
    # prefill and decoding): TTFT SLOs relative to the all-resident prefill iteration ------------
    if a.full and a.prefill_slo_points:
        se.place(0)
        # a prefill of many seconds (the 70B shape: 17 s) gets one all-resident run, one profiling pass and one
        # SLO point under the paper's schedule; the progress lines keep a long silence from looking like a hang
        heavy = pre0["iter_ns"] > 5e9
        log(f"[bench] prefill phase: all-resident prefill{' (long: one SLO point, one profiling pass)' if heavy else ''}")
        ttft0 = float(min(d["iter_ns"] for d in run_prefill(se, sn, w, x_pre, y_pre, 1 if heavy else 2)))
        log(f"[bench] prefill phase: TTFT all-resident {ttft0 / 1e6:.1f} ms; profiling the layers")
        tcp, txp = sn.sn_profile_layers(se.ctx, L, True, B, p_mean, reps=1 if heavy else 3)
        rho_p = float(np.median(txp) / np.median(tcp))
        log(f"[bench] prefill phase: layer compute {np.median(tcp) / 1e3:.0f} us, transfer {np.median(txp) / 1e3:.0f} us, rho {rho_p:.2f}")

        def prefill_point(f, sched, label):
            """Pick for TTFT SLO f x the all-resident prefill, run, check every iteration; an interval whose
            measured iterations miss the SLO is replaced by the next one that offloads fewer layers and run
            again (the analyzer's prediction leaves out what a busy link and the fences cost)."""
            slo_f = int(f * ttft0)
            try:
                n_f = sn.sn_pick_interval_from_times_sched(tcp, txp, int(slo_f * (1.0 - a.prefill_guard)), L + 1, sched)
            except sn.SnError:
                n_f = L + 1
            # no more pinned host memory than --host-limit-gb (weights of the offloaded layers)
            while n_f <= L and (L // n_f) * sn.sn_layer_blob_bytes(se.cshape) > a.host_limit_gb * 1e9:
                n_f += 1
            first = int(n_f)
            for _ in range(4):
                log(f"[bench] prefill SLO {f}x{label}: running N={n_f}")
                se.place(n_f)
                pst = run_prefill(se, sn, w, x_pre, y_pre, 2 if heavy else 3)[1:]
                pit = np.array([d["iter_ns"] for d in pst], dtype=np.float64)
                k_f = int(pst[-1]["n_offloaded"])
                if (pit <= slo_f).all() or k_f == 0:
                    break
                n_next = n_f + 1
                while n_next <= L and L // n_next >= k_f:
                    n_next += 1
                log(f"[bench] prefill SLO {f}x{label}: N={n_f} measured {pit.max() / 1e6:.2f} ms > SLO, trying N={n_next}")
                n_f = n_next
            ph = sum(d["h2d_ns"] for d in pst)
            pb = sum(d["h2d_bytes"] for d in pst)
            ps = sum(d["stall_ns"] for d in pst)
            pred, _ = sn.sn_timeline_sched(tcp, txp, n_f, sched)
            pt = {"slo_factor": f, "slo_ms": slo_f / 1e6, "picked_interval": int(n_f),
                  "picker_first_choice": first, "adjusted_after_measurement": bool(first != int(n_f)),
                  "n_offloaded": k_f, "ttft_ms": float(np.median(pit)) / 1e6,
                  "ttft_max_ms": float(pit.max()) / 1e6, "predicted_ms": pred / 1e6,
                  "every_iteration_within_slo": bool((pit <= slo_f).all()),
                  "hidden_fraction": (1 - ps / ph) if ph else 1.0,
                  "h2d_GBps": pb / (ph * 1e-9) / 1e9 if ph else None,
                  "host_resident_weight_GB": k_f * sn.sn_layer_blob_bytes(se.cshape) / 1e9,
                  "resident_GB": sn.sn_resident_bytes(se.ctx, n_f) / 1e9,
                  "over_cap": bool(sn.sn_resident_bytes(se.ctx, n_f) > w.hbm_budget > 0),
                  "prefill_tokens_per_s": T / (float(np.median(pit)) * 1e-9)}
            log(f"[bench] prefill SLO {f}x = {slo_f / 1e6:.2f} ms{label}: picked N={n_f} (K={k_f}, first choice N={first}), "
                f"TTFT {pt['ttft_ms']:.2f} max {pt['ttft_max_ms']:.2f} (predicted {pred / 1e6:.2f}) "
                f"within={pt['every_iteration_within_slo']} hidden {pt['hidden_fraction']:.3f} h2d {pt['h2d_GBps']}")
            return pt

        factors = [float(v) for v in a.prefill_slo_points.split(",") if v]
        if heavy:
            factors = factors[:1]
        pts = [prefill_point(f, sn.SN_SCHED_PAPER, "") for f in factors]
        # the same SLOs with loads issued as early as the two staging slots allow (copy stream kept busy: the
        # regime of the analyzer's closed form); the paper's schedule is restored afterwards
        eager = []
        if not heavy:
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_EAGER)
            eager = [prefill_point(f, sn.SN_SCHED_EAGER, ", eager schedule") for f in factors]
            sn.sn_set_schedule(se.ctx, sn.SN_SCHED_PAPER)
        out["prefill_phase"] = {"ttft_all_resident_ms": ttft0 / 1e6, "rho_transfer_over_compute": rho_p,
                                "guard_band": a.prefill_guard, "slo_points_eager_schedule": eager,
                                "layer_compute_us_median": float(np.median(tcp)) / 1e3,
                                "layer_transfer_us_median": float(np.median(txp)) / 1e3, "slo_points": pts}

    # ---- bandwidth contention on the host link (Sec. 4.5): a competing copy stream stands in for a second
    # GPU instance on the same bus; the coordinator widens this instance's interval until the two fit -------
    if a.contention > 0:
        import threading
        from paper_2502_08182_amd import sn_coord as CO
        se.place(0)
        ttft0c = float(min(d["iter_ns"] for d in run_prefill(se, sn, w, x_pre, y_pre, 2)))
        tcp2, txp2 = sn.sn_profile_layers(se.ctx, L, True, B, p_mean, reps=3)
        w_bytes = sn.sn_layer_blob_bytes(se.cshape)
        link_bps = int(w_bytes / (float(np.median(txp2)) * 1e-9))          # measured, this phase's transfers
        f_c = 1.5
        slo_c = int(f_c * ttft0c)
        try:
            n_solo = sn.sn_pick_interval_from_times(tcp2, txp2, int(slo_c * (1.0 - a.prefill_guard)), L + 1)
        except sn.SnError:
            n_solo = L + 1
        other_bps = int(a.contention * link_bps)
        chunk = 32 << 20
        src = torch.empty(chunk, dtype=torch.uint8, pin_memory=True)
        dst = torch.empty(chunk, dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()
        stop = threading.Event()
        moved = [0, 0.0]

        def competitor():
            period = chunk / other_bps
            t_begin = time.perf_counter()
            nxt = t_begin
            while not stop.is_set():
                with torch.cuda.stream(side):
                    dst.copy_(src, non_blocking=True)
                side.synchronize()
                moved[0] += chunk
                nxt += period
                lag = nxt - time.perf_counter()
                if lag > 0:
                    time.sleep(lag)
                else:
                    nxt = time.perf_counter()      # cannot keep up: do not accumulate debt
            moved[1] = time.perf_counter() - t_begin

        def measure(n, contended):
            se.place(n)
            if contended:
                stop.clear()
                moved[0], moved[1] = 0, 0.0
                th = threading.Thread(target=competitor)
                th.start()
                time.sleep(0.05)
            st_ = run_prefill(se, sn, w, x_pre, y_pre, 4)[1:]
            if contended:
                stop.set()
                th.join()
            it_ = np.array([d["iter_ns"] for d in st_], dtype=np.float64)
            hh = sum(d["h2d_ns"] for d in st_)
            hb = sum(d["h2d_bytes"] for d in st_)
            hs = sum(d["stall_ns"] for d in st_)
            return {"interval": int(n), "n_offloaded": int(st_[-1]["n_offloaded"]), "ttft_ms": float(np.median(it_)) / 1e6,
                    "ttft_max_ms": float(it_.max()) / 1e6, "within_slo": bool((it_ <= slo_c).all()),
                    "hidden_fraction": (1 - hs / hh) if hh else 1.0, "h2d_GBps": hb / (hh * 1e-9) / 1e9 if hh else None,
                    "competitor_GBps": (moved[0] / moved[1] / 1e9) if contended and moved[1] > 0 else 0.0}

        me = CO.make_instance(L, w_bytes, int(ttft0c), n_solo, L + 1)
        # the competitor as an instance with a single legal interval: one "layer" of other_bps bytes per second
        other = CO.make_instance(1, other_bps, 1_000_000_000, 1, 1)
        try:
            (n_adj, _), host_b, rate_b = CO.sn_coord_adjust([me, other], link_bps)
        except sn.SnError:
            n_adj, host_b, rate_b = L + 1, 0, other_bps
        res = {"slo_factor": f_c, "slo_ms": slo_c / 1e6, "link_GBps": link_bps / 1e9, "competitor_target_GBps": other_bps / 1e9,
               "interval_without_contention": int(n_solo), "interval_from_coordinator": int(n_adj),
               "coordinator_rate_GBps": rate_b / 1e9, "coordinator_host_GB": host_b / 1e9,
               "alone": measure(n_solo, False), "contended_at_solo_interval": measure(n_solo, True),
               "contended_at_coordinator_interval": measure(n_adj, True)}
        out["contention"] = res
        log(f"[bench] contention: link {link_bps / 1e9:.1f} GB/s, competitor {other_bps / 1e9:.1f} GB/s, TTFT SLO {slo_c / 1e6:.1f} ms; "
            f"alone N={n_solo}: {res['alone']['ttft_ms']:.1f} ms; contended N={n_solo}: "
            f"{res['contended_at_solo_interval']['ttft_ms']:.1f} ms (within={res['contended_at_solo_interval']['within_slo']}, "
            f"competitor got {res['contended_at_solo_interval']['competitor_GBps']:.1f} GB/s); coordinator N={n_adj}: "
            f"{res['contended_at_coordinator_interval']['ttft_ms']:.1f} ms (within={res['contended_at_coordinator_interval']['within_slo']}, "
            f"competitor got {res['contended_at_coordinator_interval']['competitor_GBps']:.1f} GB/s)")
        del src, dst

    # ---- fixed TPOT SLO while the KV cache grows: the interval is looked up in a performance record
    # before every iteration and the placement is changed when the answer changes (Sec. 4.2, 4.4) ----
    if a.repick > 1:
        from paper_2502_08182_amd import sn_record as R
        rec = R.sn_record_create(L, 0)
        se.place(0)
        lens = sorted({int(round(p_mean + W + i * K / (a.repick - 1))) for i in range(a.repick)})
        t_rec = time.time()
        for sq in lens:      # as sn_record_profile, but without the capacity bound: over-cap points are run and labelled
            tcr, txr = sn.sn_profile_layers(se.ctx, L, False, B, sq, reps=1)
            R.sn_record_put(rec, R.SN_PHASE_DECODE, B, sq, tcr, txr, L + 1)
        t_rec = time.time() - t_rec
        slo_abs = int(slo_ns * (1.0 - a.guard))

        def look(cur_len, refine=True):
            """The record's interval: the smallest that meets the bound, conservatively over the neighbouring cells; refined: of
            the intervals that keep as many layers on the host, the fastest on those cells' times (sn_record_lookup_refined)."""
            try:
                return (R.sn_record_lookup_refined if refine else R.sn_record_lookup)(rec, R.SN_PHASE_DECODE, B, cur_len, R.SN_SLO_ABS_NS, slo_abs)
            except sn.SnError as e:
                if e.code == sn.SN_E_INFEASIBLE:
                    return L + 1
                raise
        se.kv_reset([p + W + K + 1 for p in w.prompt_lens])
        n_cur = look(p_mean)
        se.place(n_cur)
        sn.sn_set_timing(se.ctx, 0)
        se.step_device(list(w.prompt_lens), True, x_pre, y_pre)
        ones = [1] * B
        for i in range(W):
            se.step_device(ones, False, x_dec[i % len(x_dec)], y_dec)
        se.stream.synchronize()
        its, picks, mig_ms = [], [], 0.0
        for i in range(K):
            n_i = look(p_mean + W + i)
            if n_i != n_cur:
                t0 = time.perf_counter()
                se.place(n_i)                 # synchronous; moves weights and the live KV of the layers that change side
                mig_ms += (time.perf_counter() - t0) * 1e3
                n_cur = n_i
            se.step_device(ones, False, x_dec[i % len(x_dec)], y_dec)
            its.append(sn.sn_get_stats(se.ctx).as_dict()["iter_ns"])
            picks.append(n_cur)
        runs = []
        for i, n in enumerate(picks):
            if not runs or runs[-1][1] != n:
                runs.append([i, n, 1])
            else:
                runs[-1][2] += 1
        its = np.array(its, dtype=np.float64)
        out["repick"] = {"slo_ms": slo_ns / 1e6, "record_seq_lens": lens, "record_build_s": t_rec,
                         "cell_intervals": [look(sq, refine=False) for sq in lens],
                         "cell_intervals_run": [look(sq) for sq in lens],
                         "interval_runs": [{"first_step": r[0], "interval": r[1], "steps": r[2]} for r in runs],
                         "placements_changed": len(runs) - 1, "migration_ms_total": mig_ms,
                         "tpot_median_ms": float(np.median(its)) / 1e6, "tpot_max_ms": float(its.max()) / 1e6,
                         "every_iteration_within_slo": bool((its <= slo_ns).all())}
        log(f"[bench] repick: record of {len(lens)} lengths built in {t_rec:.1f} s, cell intervals "
            f"{out['repick']['cell_intervals']}; runs {[(r[1], r[2]) for r in runs]}; TPOT median "
            f"{out['repick']['tpot_median_ms']:.3f} max {out['repick']['tpot_max_ms']:.3f} (SLO {slo_ns / 1e6:.3f}) "
            f"within={out['repick']['every_iteration_within_slo']} migration {mig_ms:.1f} ms")
        R.sn_record_destroy(rec)

    se.close()

    if not a.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
        log(f"[bench] cpu oracle: {out['cpu_baseline']['value']:.3f} tok/s on {out['cpu_baseline']['cores']} threads")
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
