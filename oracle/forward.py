"""CPU oracle of the decoder forward pass -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file.  It shares no code with the HIP path and imports nothing from it.

What it computes.  The paper describes serving as a layer-by-layer pass in which
every layer has the same structure and performs "attention computations" followed
by "MLP computations" on its input, once over the whole prompt (prefill) and then
once per generated token using cached keys and values (decoding) (Sec. 2.1).  It
does not spell the layer out; the layer below is the textbook pre-normalisation
decoder layer of the two families the paper evaluates (Sec. 5.1):

  OPT-like   : LayerNorm, biased projections, multi-head attention, GELU MLP
  LLaMA-like : RMSNorm, no biases, rotary position embedding, (grouped-query)
               attention, SwiGLU MLP

All arithmetic is float64 numpy, written out step by step with no blocking or
fusion.  The single deliberate rounding is that keys and values are rounded to the
model's 16-bit storage type when they enter the cache, because the cache format is
part of the offloaded layer state the method moves (Sec. 4.3).  The offloading
interval does not appear anywhere in this file: the result cannot depend on it.

Parity pins (tests/test_oracle_forward.py): library layer_norm / linear / gelu /
silu / scaled-dot-product attention in float64, the complex-number form of rotary
embedding, cached decode == full recompute, residual identity with zero output
projections, causality, GQA == MHA with repeated heads.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np
from scipy.special import erf as _erf   # library primitive: the error function


# ---------------------------------------------------------------------------
# storage rounding of cached K/V (own implementation; nothing shared)
# ---------------------------------------------------------------------------

def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the nearest f16 / bf16 value (ties to even), return float64."""
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    if dtype == "f16":
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        f = np.asarray(x, dtype=np.float64).astype(np.float32)
        u = f.view(np.uint32).astype(np.uint64)
        keep = u >> 16
        rem = u & 0xFFFF
        up = (rem > 0x8000) | ((rem == 0x8000) & ((keep & 1) == 1))
        keep = (keep + up.astype(np.uint64)) << 16
        return keep.astype(np.uint32).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------
# elementary pieces
# ---------------------------------------------------------------------------

def layer_norm(x, gain, shift, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased variance
    return (x - mu) / np.sqrt(var + eps) * gain + shift


def rms_norm(x, gain, eps):
    ms = (x ** 2).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def gelu(x):
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))       # exact (erf) form


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, theta):
    """Rotary embedding, half-split pairing: element i pairs with i + d/2.

    x: [..., d]; pos: integer position (scalar or broadcastable to x[..., 0]).
    Pair (a, b) = (x[i], x[i+d/2]) is rotated by angle pos * theta**(-2i/d).
    """
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta ** (-2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


# ---------------------------------------------------------------------------
# KV cache: cache[layer][seq] = {"k": [len, Hkv, d], "v": [len, Hkv, d]}
# ---------------------------------------------------------------------------

def new_cache(n_layers: int, batch: int, n_kv_heads: int, head_dim: int):
    return [[{"k": np.zeros((0, n_kv_heads, head_dim)), "v": np.zeros((0, n_kv_heads, head_dim))}
             for _ in range(batch)] for _ in range(n_layers)]


def cache_lens(cache) -> List[int]:
    return [c["k"].shape[0] for c in cache[0]]


# ---------------------------------------------------------------------------
# attention of one sequence's new tokens over its cache
# ---------------------------------------------------------------------------

def causal_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, start: int) -> np.ndarray:
    """q: [n_new, Hq, d] (new token t sits at position start + t); K, V: [len, Hkv, d]
    with len >= start + n_new.  Token at position p sees keys 0..p; scores are scaled by
    1/sqrt(d); query head i reads KV head floor(i * Hkv / Hq).  Returns [n_new, Hq, d]."""
    n_new, Hq, d = q.shape
    Hkv = K.shape[1]
    a = np.zeros((n_new, Hq, d))
    scale = 1.0 / math.sqrt(d)
    for t in range(n_new):
        p = start + t
        for i in range(Hq):
            g = (i * Hkv) // Hq
            s = (K[:p + 1, g, :] @ q[t, i, :]) * scale
            s = s - s.max()
            e = np.exp(s)
            a[t, i, :] = (e / e.sum()) @ V[:p + 1, g, :]
    return a


# ---------------------------------------------------------------------------
# one layer, one sequence
# ---------------------------------------------------------------------------

def layer_forward(shape: dict, w: Dict[str, np.ndarray], x: np.ndarray, kv: dict,
                  kv_dtype: Optional[str] = None) -> np.ndarray:
    """x: [n_new, hidden] new tokens of ONE sequence; kv: that sequence's cache for
    this layer (appended in place).  Returns the layer output [n_new, hidden]."""
    Hq, Hkv, d = shape["n_q_heads"], shape["n_kv_heads"], shape["head_dim"]
    eps = shape["norm_eps"]
    kv_dtype = shape["dtype"] if kv_dtype is None else kv_dtype
    n_new = x.shape[0]
    start = kv["k"].shape[0]
    pos = np.arange(start, start + n_new)

    # 1. first normalisation
    if shape["norm"] == "ln":
        u = layer_norm(x, w["n1g"], w["n1b"], eps)
    else:
        u = rms_norm(x, w["n1g"], eps)

    # 2. q, k, v projections (rows of wqkv: all q heads, then all k heads, then all v heads)
    qkv = u @ w["wqkv"].T
    if shape["has_bias"]:
        qkv = qkv + w["bqkv"]
    q = qkv[:, :Hq * d].reshape(n_new, Hq, d)
    k = qkv[:, Hq * d:(Hq + Hkv) * d].reshape(n_new, Hkv, d)
    v = qkv[:, (Hq + Hkv) * d:].reshape(n_new, Hkv, d)

    # 3. rotary embedding at the absolute position of each token
    if shape["rope"]:
        q = rope(q, pos[:, None], shape["rope_theta"])
        k = rope(k, pos[:, None], shape["rope_theta"])

    # 4. append to the cache (stored in the model's 16-bit type)
    kv["k"] = np.concatenate([kv["k"], round_to_storage(k, kv_dtype)], axis=0)
    kv["v"] = np.concatenate([kv["v"], round_to_storage(v, kv_dtype)], axis=0)
    K, V = kv["k"], kv["v"]

    # 5. causal softmax attention over the cached keys
    a = causal_attention(q, K, V, start)

    # 6. output projection + residual
    o = a.reshape(n_new, Hq * d) @ w["wo"].T
    if shape["has_bias"]:
        o = o + w["bo"]
    x = x + o

    # 7. second normalisation and MLP
    if shape["norm"] == "ln":
        u = layer_norm(x, w["n2g"], w["n2b"], eps)
    else:
        u = rms_norm(x, w["n2g"], eps)
    if shape["act"] == "gelu":
        m = u @ w["wu"].T
        if shape["has_bias"]:
            m = m + w["bu"]
        m = gelu(m)
    else:
        g_ = u @ w["wg"].T
        u_ = u @ w["wu"].T
        if shape["has_bias"]:
            g_ = g_ + w["bg"]
            u_ = u_ + w["bu"]
        m = silu(g_) * u_
    m = m @ w["wd"].T
    if shape["has_bias"]:
        m = m + w["bd"]

    # 8. residual
    return x + m


# ---------------------------------------------------------------------------
# one serving iteration over a batch (prefill: n_new = prompt length; decode: 1)
# ---------------------------------------------------------------------------

def step(shape: dict, layers: List[Dict[str, np.ndarray]], x_new: List[np.ndarray], cache,
         kv_dtype: Optional[str] = None) -> List[np.ndarray]:
    """One iteration, layer by layer (Sec. 2.1): x_new[b] is [n_new_b, hidden] for
    sequence b.  The cache is advanced in place.  Output: hidden states after the
    last layer, per sequence (no final norm, no vocabulary head)."""
    xs = [np.asarray(x, dtype=np.float64) for x in x_new]
    for l, w in enumerate(layers):
        xs = [layer_forward(shape, w, xs[b], cache[l][b], kv_dtype) for b in range(len(xs))]
    return xs


def run_workload(shape: dict, layers, prompt: np.ndarray, prompt_lens, decode_table: np.ndarray,
                 kv_dtype: Optional[str] = None):
    """Prefill followed by teacher-forced decode steps.

    prompt: [sum(prompt_lens), hidden] float64; decode_table: [steps, batch, hidden].
    Returns (prefill_out [sum(prompt_lens), hidden], decode_out [steps, batch, hidden])."""
    B = len(prompt_lens)
    cache = new_cache(len(layers), B, shape["n_kv_heads"], shape["head_dim"])
    offs = np.concatenate([[0], np.cumsum(prompt_lens)])
    xs = [prompt[offs[b]:offs[b + 1]] for b in range(B)]
    pre = np.concatenate(step(shape, layers, xs, cache, kv_dtype), axis=0)
    outs = []
    for t in range(decode_table.shape[0]):
        ys = step(shape, layers, [decode_table[t, b][None, :] for b in range(B)], cache, kv_dtype)
        outs.append(np.concatenate(ys, axis=0))
    dec = np.stack(outs, axis=0) if outs else np.zeros((0, B, shape["hidden"]))
    return pre, dec
