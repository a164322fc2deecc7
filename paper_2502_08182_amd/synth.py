"""Seeded synthetic workloads: model shapes, random weights, hidden-state inputs.

This module only *generates and formats data*.  It holds none of the method's
arithmetic (no norm, GEMM, attention, placement, timeline or picker code) and is
the one module that both the CPU oracle's tests and the HIP path's tests use, so
that the two sides see identical bits.  It imports neither of them.

The paper evaluates with a random dataloader (custom batch size and sequence
length) and states that results do not depend on content (Sec. 5.1, Workload);
the shapes below follow the decoder-only families the paper evaluates (Sec. 5.1,
OPT / LLaMA style layers: attention followed by an MLP, Sec. 2.1).

16-bit storage convention: every tensor is a numpy uint16 array of raw bit
patterns plus a dtype tag ("f16" or "bf16"); `widen` turns it into float64.
"""
from __future__ import annotations

from dataclasses import dataclass, field, asdict
from typing import Dict, List, Tuple

import numpy as np

# ----------------------------------------------------------------------------
# 16-bit formats (storage only)
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array once to the 16-bit storage type; returns uint16 bits."""
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored 16-bit values to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# Model shape
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    act: str = "gelu"        # "gelu" | "swiglu"
    norm: str = "ln"         # "ln" | "rms"
    rope: bool = False
    has_bias: bool = True
    dtype: str = "f16"       # "f16" | "bf16"
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0

    def as_dict(self) -> dict:
        return asdict(self)

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2


def tensor_specs(s: ModelShape) -> List[Tuple[str, Tuple[int, ...]]]:
    """Canonical order and shape of one layer's tensors.

    Matrices are [out_features, in_features] row-major (y = x @ W.T + b).
    """
    qd = s.n_q_heads * s.head_dim
    specs: List[Tuple[str, Tuple[int, ...]]] = [("wqkv", (s.qkv_out, s.hidden))]
    if s.has_bias:
        specs.append(("bqkv", (s.qkv_out,)))
    specs.append(("wo", (s.hidden, qd)))
    if s.has_bias:
        specs.append(("bo", (s.hidden,)))
    if s.act == "swiglu":
        specs.append(("wg", (s.ffn, s.hidden)))
        if s.has_bias:
            specs.append(("bg", (s.ffn,)))
    specs.append(("wu", (s.ffn, s.hidden)))
    if s.has_bias:
        specs.append(("bu", (s.ffn,)))
    specs.append(("wd", (s.hidden, s.ffn)))
    if s.has_bias:
        specs.append(("bd", (s.hidden,)))
    specs.append(("n1g", (s.hidden,)))
    if s.norm == "ln":
        specs.append(("n1b", (s.hidden,)))
    specs.append(("n2g", (s.hidden,)))
    if s.norm == "ln":
        specs.append(("n2b", (s.hidden,)))
    return specs


BLOB_ALIGN = 256  # bytes; every tensor of the caller-side layer blob starts on this boundary


def blob_layout(s: ModelShape) -> Tuple[Dict[str, Tuple[int, Tuple[int, ...]]], int]:
    """Byte offset of every tensor in the caller-side layer blob, and its total size."""
    off = 0
    out: Dict[str, Tuple[int, Tuple[int, ...]]] = {}
    for name, shp in tensor_specs(s):
        out[name] = (off, shp)
        n = int(np.prod(shp)) * 2
        off += (n + BLOB_ALIGN - 1) // BLOB_ALIGN * BLOB_ALIGN
    return out, off


def make_layer(s: ModelShape, layer: int, seed: int = 0) -> Dict[str, np.ndarray]:
    """One layer's tensors as uint16 bit arrays.

    Matrices and biases ~ N(0, 0.02^2); norm gains 1 + N(0, 0.02^2); norm shifts
    N(0, 0.02^2); each rounded once to the storage dtype.
    """
    rng = np.random.default_rng([int(seed), int(layer)])
    out: Dict[str, np.ndarray] = {}
    for name, shp in tensor_specs(s):
        v = rng.standard_normal(shp, dtype=np.float32) * np.float32(0.02)
        if name in ("n1g", "n2g"):
            v = v + np.float32(1.0)
        out[name] = to_bits(v, s.dtype)
    return out


def pack_blob(s: ModelShape, tensors: Dict[str, np.ndarray]) -> np.ndarray:
    """Caller-side layer blob (uint8) in the canonical order."""
    lay, total = blob_layout(s)
    blob = np.zeros(total, dtype=np.uint8)
    for name, (off, shp) in lay.items():
        t = np.ascontiguousarray(tensors[name], dtype=np.uint16)
        assert t.shape == tuple(shp), (name, t.shape, shp)
        b = t.reshape(-1).view(np.uint8)
        blob[off:off + b.size] = b
    return blob


def widen_layer(s: ModelShape, tensors: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: widen(v, s.dtype) for k, v in tensors.items()}


# ----------------------------------------------------------------------------
# Workloads
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    batch: int
    prompt_lens: Tuple[int, ...]
    decode_steps: int
    hbm_budget: int = 0          # bytes; 0 = no cap
    intervals: Tuple[int, ...] = ()
    slo_factors: Tuple[float, ...] = ()
    note: str = ""

    @property
    def max_seq(self) -> int:
        return max(self.prompt_lens) + self.decode_steps


def make_prompt(w: Workload, seed: int = 1) -> np.ndarray:
    """Prefill hidden states [sum(prompt_lens), hidden] ~ N(0,1), as 16-bit bits."""
    rng = np.random.default_rng([int(seed), 0])
    t = int(sum(w.prompt_lens))
    return to_bits(rng.standard_normal((t, w.shape.hidden), dtype=np.float32), w.shape.dtype)


def make_decode_table(w: Workload, seed: int = 2) -> np.ndarray:
    """Teacher-forced decode inputs [decode_steps, batch, hidden] ~ N(0,1), 16-bit bits."""
    rng = np.random.default_rng([int(seed), 0])
    return to_bits(
        rng.standard_normal((w.decode_steps, w.batch, w.shape.hidden), dtype=np.float32),
        w.shape.dtype)


def _opt(L, h, heads, ffn, dtype="f16") -> ModelShape:
    return ModelShape(L, h, heads, heads, h // heads, ffn, act="gelu", norm="ln", rope=False,
                      has_bias=True, dtype=dtype)


def _llama(L, h, hq, hkv, ffn, dtype="bf16") -> ModelShape:
    return ModelShape(L, h, hq, hkv, h // hq, ffn, act="swiglu", norm="rms", rope=True,
                      has_bias=False, dtype=dtype)


GB = 10 ** 9


def _c4_prompts(batch: int, seed: int = 3) -> Tuple[int, ...]:
    rng = np.random.default_rng([int(seed), 0])
    return tuple(int(v) for v in rng.integers(256, 2049, size=batch))


def workload(name: str, **over) -> Workload:
    """The five configurations this build measures or checks, plus truncated
    instances of the large ones (same per-layer shape, few layers, small batch)
    that the CPU oracle can finish in seconds."""
    if name == "c1":      # tiny plumbing-scale decoder
        w = Workload("c1", _opt(4, 256, 4, 1024), 2, (32, 32), 8, 0, (2,), ())
    elif name == "c2":    # OPT-6.7B shape
        w = Workload("c2", _opt(32, 4096, 32, 16384), 8, (512,) * 8, 32, 8 * GB,
                     (2, 3, 4, 6, 8), (2.0,))
    elif name == "c3":    # Llama-2-13B shape
        w = Workload("c3", _llama(40, 5120, 40, 40, 13824), 32, (1024,) * 32, 64, 20 * GB,
                     (), (1.2, 1.5, 2.0))
    elif name == "c4":    # OPT-30B shape, ragged prompts
        b = int(over.pop("batch", 8))
        w = Workload("c4", _opt(48, 7168, 56, 28672), b, _c4_prompts(b), 128, 40 * GB, (), (2.0,))
    elif name == "c5":    # Llama-2-70B shape, GQA
        w = Workload("c5", _llama(80, 8192, 64, 8, 28672), 64, (2048,) * 64, 128, 96 * GB,
                     (), (2.0,))
    elif name == "c2t":   # truncated: real per-layer shape of c2
        w = Workload("c2t", _opt(2, 4096, 32, 16384), 2, (96, 37), 2, 0, (2,), ())
    elif name == "c3t":
        w = Workload("c3t", _llama(2, 5120, 40, 40, 13824), 2, (80, 33), 2, 0, (2,), ())
    elif name == "c4t":
        w = Workload("c4t", _opt(1, 7168, 56, 28672), 2, (48, 21), 2, 0, (1,), ())
    elif name == "c5t":
        w = Workload("c5t", _llama(2, 8192, 64, 8, 28672), 2, (72, 19), 2, 0, (2,), ())
    else:
        raise KeyError(name)
    if over:
        from dataclasses import replace
        w = replace(w, **over)
    return w
