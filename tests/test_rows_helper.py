"""The full-size GPU parity tests check sampled rows against pieces of the oracle composed per row
(tests/test_gpu_e2e.py::_layer_rows).  This pins that composition, on the CPU, to the oracle's own
layer_forward on a small sequence, for both layer families."""
import numpy as np

from oracle import forward as ofw
from paper_2502_08182_amd import synth
from tests.test_gpu_e2e import _layer_rows


def test_rows_helper_equals_the_oracle_layer():
    shapes = [synth.ModelShape(1, 128, 4, 2, 64, 256, act="swiglu", norm="rms", rope=True, has_bias=False, dtype="bf16"),
              synth.ModelShape(1, 128, 2, 2, 64, 256, act="gelu", norm="ln", rope=False, has_bias=True, dtype="f16")]
    for s in shapes:
        layer = synth.make_layer(s, 0, 0)
        x = np.random.default_rng(0).standard_normal((20, s.hidden))
        empty = {"k": np.zeros((0, s.n_kv_heads, s.head_dim)), "v": np.zeros((0, s.n_kv_heads, s.head_dim))}
        full = ofw.layer_forward(s.as_dict(), synth.widen_layer(s, layer), x, empty, "f16")
        rows = [0, 3, 19]
        assert np.abs(_layer_rows(s, layer, x, rows) - full[rows]).max() <= 1e-12
