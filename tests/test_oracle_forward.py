"""Pins for oracle/forward.py against things that are not the oracle itself:
library routines (torch float64 layer_norm / linear / gelu / silu / scaled dot product
attention), the complex-number form of rotary embedding, closed forms and invariants.
Each is chosen so that a plausible slip (dropped term, transposed operand, wrong head
mapping, wrong sign, off-by-one in the causal mask) fails at least one test."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import forward as ofw
from paper_2502_08182_amd import synth

torch.set_num_threads(4)


def _shape(**kw):
    base = dict(n_layers=2, hidden=48, n_q_heads=4, n_kv_heads=4, head_dim=12, ffn=80,
                act="gelu", norm="ln", rope=False, has_bias=True, dtype="f16")
    base.update(kw)
    return synth.ModelShape(**base)


def _layers(s, seed=0, scale=8.0):
    # larger weights than the workloads use, so that every term matters numerically
    out = []
    for l in range(s.n_layers):
        w = synth.widen_layer(s, synth.make_layer(s, l, seed))
        for k in w:
            if k.startswith("w") or k.startswith("b"):
                w[k] = w[k] * scale
        out.append(w)
    return out


def _torch_layer_prefill(s, w, x):
    """Textbook layer from torch library routines, float64, one sequence from an empty cache."""
    T = x.shape[0]
    tw = {k: torch.from_numpy(v) for k, v in w.items()}
    x = torch.from_numpy(x)
    Hq, Hkv, d = s.n_q_heads, s.n_kv_heads, s.head_dim

    def norm(x, g, b):
        if s.norm == "ln":
            return F.layer_norm(x, (s.hidden,), g, b, s.norm_eps)
        return F.rms_norm(x, (s.hidden,), g, s.norm_eps)

    u = norm(x, tw["n1g"], tw.get("n1b"))
    qkv = F.linear(u, tw["wqkv"], tw.get("bqkv"))
    q, k, v = torch.split(qkv, [Hq * d, Hkv * d, Hkv * d], dim=-1)
    q = q.view(T, Hq, d).transpose(0, 1)
    k = k.view(T, Hkv, d).transpose(0, 1)
    v = v.view(T, Hkv, d).transpose(0, 1)
    if s.rope:
        pos = torch.arange(T, dtype=torch.float64)
        inv = s.rope_theta ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
        rot = torch.polar(torch.ones(T, d // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

        def cplx(t):  # half-split pairing as complex numbers
            z = torch.complex(t[..., : d // 2], t[..., d // 2:]) * rot
            return torch.cat([z.real, z.imag], dim=-1)
        q, k = cplx(q), cplx(k)
    rep = Hq // Hkv
    a = F.scaled_dot_product_attention(q[None], k.repeat_interleave(rep, 0)[None],
                                       v.repeat_interleave(rep, 0)[None], is_causal=True)[0]
    a = a.transpose(0, 1).reshape(T, Hq * d)
    x = x + F.linear(a, tw["wo"], tw.get("bo"))
    u = norm(x, tw["n2g"], tw.get("n2b"))
    if s.act == "gelu":
        m = F.gelu(F.linear(u, tw["wu"], tw.get("bu")))
    else:
        m = F.silu(F.linear(u, tw["wg"], tw.get("bg"))) * F.linear(u, tw["wu"], tw.get("bu"))
    return (x + F.linear(m, tw["wd"], tw.get("bd"))).numpy()


FAMILIES = {
    "opt": dict(),
    "llama": dict(act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16"),
    "llama_gqa": dict(act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16",
                      n_q_heads=8, n_kv_heads=2, head_dim=6),
    "mixed": dict(act="swiglu", norm="ln", rope=True, has_bias=True),
}


@pytest.mark.parametrize("fam", list(FAMILIES))
def test_layer_matches_torch_library_float64(fam):
    s = _shape(**FAMILIES[fam])
    rng = np.random.default_rng(5)
    layers = _layers(s)
    x = rng.standard_normal((11, s.hidden))
    want = x
    for w in layers:
        want = _torch_layer_prefill(s, w, want)
    cache = ofw.new_cache(s.n_layers, 1, s.n_kv_heads, s.head_dim)
    got = ofw.step(s.as_dict(), layers, [x], cache, kv_dtype="f64")[0]
    assert np.abs(got - want).max() <= 1e-11 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("fam", list(FAMILIES))
def test_cached_decode_equals_full_recompute(fam):
    s = _shape(**FAMILIES[fam])
    rng = np.random.default_rng(6)
    layers = _layers(s)
    x = rng.standard_normal((9, s.hidden))
    full = ofw.step(s.as_dict(), layers, [x], ofw.new_cache(s.n_layers, 1, s.n_kv_heads, s.head_dim),
                    kv_dtype="f64")[0]
    cache = ofw.new_cache(s.n_layers, 1, s.n_kv_heads, s.head_dim)
    got = [ofw.step(s.as_dict(), layers, [x[:4]], cache, kv_dtype="f64")[0]]
    got.append(ofw.step(s.as_dict(), layers, [x[4:6]], cache, kv_dtype="f64")[0])   # chunk of 2
    for t in range(6, 9):
        got.append(ofw.step(s.as_dict(), layers, [x[t:t + 1]], cache, kv_dtype="f64")[0])
    got = np.concatenate(got, axis=0)
    assert ofw.cache_lens(cache) == [9]
    assert np.abs(got - full).max() <= 1e-11 * np.abs(full).max()


def test_prefill_of_one_token_is_decode_from_empty_cache_and_attends_to_itself():
    s = _shape()
    layers = _layers(s)
    x = np.random.default_rng(7).standard_normal((1, s.hidden))
    y = ofw.step(s.as_dict(), layers, [x], ofw.new_cache(2, 1, 4, 12), kv_dtype="f64")[0]
    # with one key softmax is 1 -> attention output is v itself: check layer 0 by hand
    w = layers[0]
    u = F.layer_norm(torch.from_numpy(x), (s.hidden,), torch.from_numpy(w["n1g"]),
                     torch.from_numpy(w["n1b"]), s.norm_eps).numpy()
    v = (u @ w["wqkv"].T + w["bqkv"])[:, -s.n_kv_heads * s.head_dim:]
    x1 = x + v @ w["wo"].T + w["bo"]
    c = ofw.new_cache(1, 1, 4, 12)
    ofw.step(s.as_dict(), layers[:1], [x], c, kv_dtype="f64")
    # the part before the MLP is recoverable: out - mlp(x1) == x1
    s1 = s.as_dict()
    out0 = ofw.step(s1, layers[:1], [x], ofw.new_cache(1, 1, 4, 12), kv_dtype="f64")[0]
    u2 = F.layer_norm(torch.from_numpy(x1), (s.hidden,), torch.from_numpy(w["n2g"]),
                      torch.from_numpy(w["n2b"]), s.norm_eps)
    mlp = F.linear(F.gelu(F.linear(u2, torch.from_numpy(w["wu"]), torch.from_numpy(w["bu"]))),
                   torch.from_numpy(w["wd"]), torch.from_numpy(w["bd"])).numpy()
    assert np.abs(out0 - (x1 + mlp)).max() < 1e-11
    assert y.shape == (1, s.hidden)


@pytest.mark.parametrize("fam", ["opt", "llama"])
def test_residual_identity_when_output_projections_are_zero(fam):
    s = _shape(**FAMILIES[fam])
    layers = _layers(s)
    for w in layers:
        w["wo"][:] = 0
        w["wd"][:] = 0
        for b in ("bo", "bd"):
            if b in w:
                w[b][:] = 0
    x = np.random.default_rng(8).standard_normal((5, s.hidden))
    y = ofw.step(s.as_dict(), layers, [x], ofw.new_cache(2, 1, s.n_kv_heads, s.head_dim))[0]
    assert np.array_equal(y, x)


def test_causality_future_tokens_do_not_change_earlier_outputs():
    s = _shape(**FAMILIES["llama"])
    layers = _layers(s)
    rng = np.random.default_rng(9)
    x = rng.standard_normal((8, s.hidden))
    x2 = x.copy()
    x2[5:] = rng.standard_normal((3, s.hidden))
    mk = lambda: ofw.new_cache(2, 1, s.n_kv_heads, s.head_dim)
    a = ofw.step(s.as_dict(), layers, [x], mk(), kv_dtype="f64")[0]
    b = ofw.step(s.as_dict(), layers, [x2], mk(), kv_dtype="f64")[0]
    assert np.array_equal(a[:5], b[:5])
    assert np.abs(a[5:] - b[5:]).max() > 1e-3


def test_sequences_in_a_batch_are_independent():
    s = _shape()
    layers = _layers(s)
    rng = np.random.default_rng(10)
    xa, xb = rng.standard_normal((6, s.hidden)), rng.standard_normal((3, s.hidden))
    both = ofw.step(s.as_dict(), layers, [xa, xb], ofw.new_cache(2, 2, 4, 12))
    solo = ofw.step(s.as_dict(), layers, [xb], ofw.new_cache(2, 1, 4, 12))
    assert np.array_equal(both[1], solo[0])


def test_gqa_equals_mha_with_repeated_kv_heads():
    g = _shape(**FAMILIES["llama_gqa"])
    m = _shape(**dict(FAMILIES["llama_gqa"], n_kv_heads=8))
    gl = _layers(g)
    ml = []
    d, Hq, Hkv = g.head_dim, g.n_q_heads, g.n_kv_heads
    for w in gl:
        w2 = dict(w)
        wq = w["wqkv"][:Hq * d]
        wk = w["wqkv"][Hq * d:(Hq + Hkv) * d].reshape(Hkv, d, -1)
        wv = w["wqkv"][(Hq + Hkv) * d:].reshape(Hkv, d, -1)
        rep = Hq // Hkv
        w2["wqkv"] = np.concatenate([wq, np.repeat(wk, rep, axis=0).reshape(Hq * d, -1),
                                     np.repeat(wv, rep, axis=0).reshape(Hq * d, -1)], axis=0)
        ml.append(w2)
    x = np.random.default_rng(11).standard_normal((7, g.hidden))
    a = ofw.step(g.as_dict(), gl, [x], ofw.new_cache(2, 1, 2, d), kv_dtype="f64")[0]
    b = ofw.step(m.as_dict(), ml, [x], ofw.new_cache(2, 1, 8, d), kv_dtype="f64")[0]
    assert np.abs(a - b).max() <= 1e-12 * np.abs(a).max()


def test_rope_properties():
    rng = np.random.default_rng(12)
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    assert np.array_equal(ofw.rope(q, 0, 10000.0), q)                      # position 0: identity
    for p in (1, 17, 300):
        assert abs(np.linalg.norm(ofw.rope(q, p, 10000.0)) - np.linalg.norm(q)) < 1e-12
    # scores depend on the position difference only
    a = ofw.rope(q, 40, 10000.0) @ ofw.rope(k, 33, 10000.0)
    b = ofw.rope(q, 107, 10000.0) @ ofw.rope(k, 100, 10000.0)
    assert abs(a - b) < 1e-10
    # first pair rotates by exactly `pos` radians (frequency theta^0 = 1); pairs are (i, i+d/2)
    e = np.zeros(16)
    e[0] = 1.0
    r = ofw.rope(e, 2, 10000.0)
    assert abs(r[0] - math.cos(2.0)) < 1e-15 and abs(r[8] - math.sin(2.0)) < 1e-15
    assert np.count_nonzero(r) == 2
    # last pair's frequency is theta^(-(d-2)/d)
    e = np.zeros(16)
    e[7] = 1.0
    r = ofw.rope(e, 5, 10000.0)
    ang = 5 * 10000.0 ** (-14.0 / 16.0)
    assert abs(r[7] - math.cos(ang)) < 1e-15 and abs(r[15] - math.sin(ang)) < 1e-15


def test_pointwise_closed_forms():
    assert ofw.gelu(np.array([0.0]))[0] == 0.0
    # gelu(x) = x * Phi(x); Phi(1) = 0.841344746068543 (standard normal CDF)
    assert abs(ofw.gelu(np.array([1.0]))[0] - 0.841344746068543) < 1e-14
    assert abs(ofw.gelu(np.array([-1.0]))[0] + (1 - 0.841344746068543)) < 1e-14
    xs = np.linspace(-6, 6, 41)
    want = np.array([0.5 * x * (1 + math.erf(x / math.sqrt(2))) for x in xs])
    assert np.abs(ofw.gelu(xs) - want).max() < 1e-15
    assert abs(ofw.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15
    assert ofw.silu(np.array([0.0]))[0] == 0.0


def test_norm_closed_forms():
    rng = np.random.default_rng(13)
    x = rng.standard_normal((3, 64)) * 5 + 2
    y = ofw.layer_norm(x, np.ones(64), np.zeros(64), 0.0)
    assert np.abs(y.mean(-1)).max() < 1e-13 and np.abs(y.var(-1) - 1).max() < 1e-12
    y = ofw.rms_norm(x, np.ones(64), 0.0)
    assert np.abs((y ** 2).mean(-1) - 1).max() < 1e-12
    # constant row: LN gives the shift, RMS gives sign * gain
    c = np.full((1, 8), 3.0)
    assert np.allclose(ofw.layer_norm(c, np.full(8, 2.0), np.full(8, 0.5), 1e-5), 0.5)
    assert np.allclose(ofw.rms_norm(c, np.full(8, 2.0), 0.0), 2.0)


@pytest.mark.parametrize("dtype,tdtype", [("f16", torch.float16), ("bf16", torch.bfloat16)])
def test_storage_rounding_matches_torch_and_generator(dtype, tdtype):
    rng = np.random.default_rng(14)
    x = np.concatenate([rng.standard_normal(4096) * 3, [0.0, 1.0, -1.0, 1 + 2 ** -8, 1 + 3 * 2 ** -9,
                        1 + 2 ** -11, 1 + 3 * 2 ** -12, 65504.0, 1e-7]]).astype(np.float32)
    got = ofw.round_to_storage(x.astype(np.float64), dtype)
    want = torch.from_numpy(x).to(tdtype).to(torch.float64).numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(synth.widen(synth.to_bits(x, dtype), dtype), want)


def test_config1_oracle_is_finite_and_kv_rounding_is_small():
    w = synth.workload("c1")
    s = w.shape
    layers = [synth.widen_layer(s, synth.make_layer(s, l, 0)) for l in range(s.n_layers)]
    prompt = synth.widen(synth.make_prompt(w), s.dtype)
    table = synth.widen(synth.make_decode_table(w), s.dtype)
    pre, dec = ofw.run_workload(s.as_dict(), layers, prompt, w.prompt_lens, table)
    pre64, dec64 = ofw.run_workload(s.as_dict(), layers, prompt, w.prompt_lens, table, kv_dtype="f64")
    assert pre.shape == (64, 256) and dec.shape == (8, 2, 256)
    assert np.isfinite(pre).all() and np.isfinite(dec).all()
    rms = math.sqrt((dec64 ** 2).mean())
    assert np.abs(dec - dec64).max() <= 1e-3 * rms       # storing K/V in f16 barely matters
    assert np.abs(dec - dec64).max() > 0                  # ... but it is applied
