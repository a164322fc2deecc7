"""Convenience driver around the C ABI: owns a context, device buffers and a stream.

It only marshals: uploads 16-bit bit patterns, calls sn_* and downloads results.
PyTorch supplies device memory and the stream, nothing else.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import sn, synth


def _dev_bits(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def _host_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class Session:
    def __init__(self, shape: synth.ModelShape, max_batch: int, max_seq: int, max_tokens: int = 0,
                 hbm_budget: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path cannot run (there is no CPU fallback)")
        self.ms = shape
        self.cshape = sn.make_shape(shape, max_batch, max_seq, max_tokens)
        self.stream = torch.cuda.Stream()
        self.ctx = sn.sn_init(self.cshape, hbm_budget, self.stream.cuda_stream)
        self.L = shape.n_layers
        self.kv_len: Optional[np.ndarray] = None

    def close(self):
        if self.ctx is not None:
            sn.sn_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    # -- weights ------------------------------------------------------------------
    def load_synthetic_weights(self, seed: int = 0, layers: Optional[Sequence[dict]] = None):
        for l in range(self.L):
            t = layers[l] if layers is not None else synth.make_layer(self.ms, l, seed)
            sn.sn_set_layer_weights(self.ctx, l, synth.pack_blob(self.ms, t))

    def load_device_generated_weights(self, seed: int = 0, distinct: int = 0):
        """Random N(0, 0.02) weights drawn on the GPU with torch (plumbing), for shapes too
        large to generate on the host quickly.  distinct > 0: only that many different
        layer blobs are drawn and reused cyclically."""
        lay, total = synth.blob_layout(self.ms)
        tdt = torch.bfloat16 if self.ms.dtype == "bf16" else torch.float16
        g = torch.Generator(device="cuda")
        cache = {}
        for l in range(self.L):
            key = l % distinct if distinct else l
            if key not in cache:
                g.manual_seed(seed * 1000003 + key)
                blob = torch.zeros(total // 2, dtype=torch.int16, device="cuda")
                for name, (off, shp) in lay.items():
                    n = int(np.prod(shp))
                    v = torch.randn(n, generator=g, device="cuda", dtype=torch.float32) * 0.02
                    if name in ("n1g", "n2g"):
                        v = v + 1.0
                    blob[off // 2: off // 2 + n] = v.to(tdt).view(torch.int16)
                if not distinct:
                    cache.clear()
                cache[key] = blob.cpu().numpy()
            sn.sn_set_layer_weights(self.ctx, l, cache[key])

    # -- placement / kv ------------------------------------------------------------
    def place(self, N: int):
        sn.sn_place(self.ctx, N)

    def kv_reset(self, capacity: Sequence[int]):
        sn.sn_kv_reset(self.ctx, capacity)
        self.kv_len = np.zeros(len(capacity), dtype=np.int32)

    def kv_truncate(self, length: Sequence[int]):
        sn.sn_kv_truncate(self.ctx, length)
        self.kv_len[:] = np.asarray(length, dtype=np.int32)

    # -- iterations ------------------------------------------------------------------
    def step_device(self, n_new: Sequence[int], is_prefill: bool, hidden_in: torch.Tensor,
                    hidden_out: torch.Tensor):
        sn.sn_step(self.ctx, n_new, is_prefill, hidden_in, self.kv_len, hidden_out)

    def step(self, n_new: Sequence[int], is_prefill: bool, hidden_bits: np.ndarray, want_f32: bool = False):
        """hidden_bits: uint16 [sum n_new, hidden]; returns the output as uint16 bits
        (and, if want_f32, also the fp32 hidden states before the final rounding)."""
        with torch.cuda.stream(self.stream):
            x = _dev_bits(hidden_bits)
            y = torch.empty_like(x)
            f = torch.empty(hidden_bits.shape, dtype=torch.float32, device="cuda") if want_f32 else None
            self.stream.synchronize()
            self.step_device(n_new, is_prefill, x, y)
            if want_f32:
                sn.sn_read_hidden_f32(self.ctx, f, f.numel() * 4)
            self.stream.synchronize()
            out = _host_bits(y).reshape(hidden_bits.shape)
            return (out, f.cpu().numpy()) if want_f32 else out

    def run_workload(self, w: synth.Workload, prompt_bits: np.ndarray, table_bits: np.ndarray, want_f32: bool = False):
        """Prefill then teacher-forced decode; returns (prefill_out_bits, decode_out_bits)
        [, prefill_f32, decode_f32]."""
        self.kv_reset([p + w.decode_steps for p in w.prompt_lens])
        pre = self.step(list(w.prompt_lens), True, prompt_bits, want_f32)
        outs = [self.step([1] * w.batch, False, table_bits[t], want_f32) for t in range(table_bits.shape[0])]
        if not want_f32:
            dec = np.stack(outs, axis=0) if outs else np.zeros((0, w.batch, self.ms.hidden), dtype=np.uint16)
            return pre, dec
        dec = np.stack([o[0] for o in outs], axis=0)
        return pre[0], dec, pre[1], np.stack([o[1] for o in outs], axis=0)

    def stats(self) -> dict:
        return sn.sn_get_stats(self.ctx).as_dict()
