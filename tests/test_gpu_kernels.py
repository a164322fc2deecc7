"""GPU parity of each layer kernel against the matching piece of the CPU oracle, through
the per-kernel C ABI.  Sizes span several tiles and ragged tails.

The bar, per element: |got - want| <= C_ARITH x RMS(want) + HALF_ULP x |want|.
  * HALF_ULP x |want| is the one rounding every kernel must make, to its output type: at most
    half an ulp of the element, 2^-11 |v| for float16, 2^-8 |v| for bfloat16, nothing for an
    fp32 output.  It has to be per element: for bfloat16 it alone reaches 1.6e-2 x RMS on an
    element of 4 x RMS, and activation outputs (GELU, SwiGLU) have heavier tails than that.
  * C_ARITH x RMS is everything else the kernel may add: fp32 accumulation in another order
    (~1e-6), and the 16-bit roundings inside the attention kernels (rotated q and the softmax
    weights are rounded to the storage type before the matrix-core products: relative 2^-12 /
    2^-9 per term, which over a row of weights comes to about 1e-4 / 1e-3 x RMS typically and
    four times that at the worst element of a tensor).  2e-3 for float16 and 8e-3 for
    bfloat16 leave a factor of two over that model and stay 10x / 2.5x inside the
    end-to-end bar of 2e-2 x RMS, which is asserted as well wherever the output rounding
    alone cannot exceed it (float16 and fp32 outputs)."""
import math

import numpy as np
import pytest
import torch

from oracle import forward as ofw
from paper_2502_08182_amd import sn, synth
from paper_2502_08182_amd import sn_kernels as K

pytestmark = pytest.mark.gpu

DT = {"f16": sn.SN_F16, "bf16": sn.SN_BF16}
C_ARITH = {"f16": 2e-3, "bf16": 8e-3}                      # x RMS(expected)
# Attention: a query that sees one or two keys passes the rounding of its softmax weights and of its rotated q
# (2^-12 relative in float16, 2^-9 in bfloat16, each) on undiminished, times values of up to 4 x RMS:
# 2 * 2^-9 * 4 = 1.6e-2 x RMS for bfloat16 (measured 1.4e-2), an eighth of that for float16 (measured 1.0e-3).
C_ATTN = {"f16": 2.5e-3, "bf16": 2e-2}                     # x RMS(expected row)
HALF_ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8, "f32": 0.0}   # x |expected element|, by output type
E2E_BAR = 2e-2                                              # x RMS(expected)


def dev16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def host16(t):
    return t.cpu().numpy().view(np.uint16)


def rms(a):
    return math.sqrt(float((np.asarray(a, dtype=np.float64) ** 2).mean()))


def check(got, want, dtype, what, out="same", want_is_rounded=False, per_row=False, bar=None):
    """dtype: the 16-bit type the kernel computes with; out: its output type ("same", or "f32").
    want_is_rounded: the expected values were themselves rounded to the output type (a cache row), so a value
    that lands on the other side of a rounding boundary differs by a whole ulp, not half of one.
    per_row: RMS taken over each row (last axis) instead of the whole tensor -- for attention outputs, whose
    rows are averages over very different numbers of keys (a query that sees 2 keys has values of the size of
    V, one that sees 500 has values 20 times smaller) while the error of a row scales with its own values."""
    out = dtype if out == "same" else out
    bar = C_ARITH[dtype] if bar is None else bar
    want = np.asarray(want, dtype=np.float64)
    r = np.sqrt((want ** 2).mean(axis=-1, keepdims=True)) if per_row else rms(want)
    d = np.abs(got - want)
    arith = float(((d - (2.0 if want_is_rounded else 1.0) * HALF_ULP[out] * np.abs(want)) / r).max())   # beyond the output rounding
    print(f"{what}: max|d| = {(d / r).max():.2e} x RMS, beyond output rounding {max(arith, 0.0):.2e} x RMS "
          f"(bar {bar:.1e}), max|want| = {(np.abs(want) / r).max():.1f} x RMS{' (per row)' if per_row else ''}", flush=True)
    assert np.isfinite(got).all(), what
    assert arith <= bar, (what, arith)
    if out != "bf16":
        assert (d / r).max() <= E2E_BAR, (what, (d / r).max())


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("is_ln", [True, False])
def test_norm(dtype, is_ln):
    rng = np.random.default_rng(1)
    T, h = 37, 1184
    x = (rng.standard_normal((T, h)) * 3 + 0.5).astype(np.float32)
    g = synth.to_bits(1 + 0.1 * rng.standard_normal(h), dtype)
    b = synth.to_bits(0.1 * rng.standard_normal(h), dtype)
    out = torch.zeros(T, h, dtype=torch.int16, device="cuda")
    K.sn_k_norm(DT[dtype], is_ln, torch.from_numpy(x).cuda(), dev16(g), dev16(b), out, T, h, 1e-5)
    torch.cuda.synchronize()
    got = synth.widen(host16(out), dtype)
    x64 = x.astype(np.float64)
    want = (ofw.layer_norm(x64, synth.widen(g, dtype), synth.widen(b, dtype), 1e-5) if is_ln
            else ofw.rms_norm(x64, synth.widen(g, dtype), 1e-5))
    check(got, want, dtype, f"norm ln={is_ln}")


def _gemm_case(dtype, path, epi, M, N, Kd, bias, seed):
    rng = np.random.default_rng(seed)
    Wrows = 2 * N if epi == K.EPI_SWIGLU16 else N
    xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
    if epi == K.EPI_SWIGLU16:
        wg = synth.to_bits(rng.standard_normal((N, Kd)) * 0.05, dtype)
        wu = synth.to_bits(rng.standard_normal((N, Kd)) * 0.05, dtype)
        tiled = np.zeros(2 * N * Kd, dtype=np.uint16)
        K.sn_k_tile_weights(wg, N, Kd, tiled, 2, 0)
        K.sn_k_tile_weights(wu, N, Kd, tiled, 2, 1)
    else:
        wb = synth.to_bits(rng.standard_normal((N, Kd)) * 0.05, dtype)
        tiled = K.sn_k_tile_weights(wb, N, Kd)
    bb = synth.to_bits(rng.standard_normal(Wrows) * 0.3, dtype) if bias else None
    x64 = synth.widen(xb, dtype)
    b64 = synth.widen(bb, dtype) if bias else np.zeros(Wrows)
    if epi == K.EPI_RESID32:
        r0 = rng.standard_normal((M, N)).astype(np.float32)
        out = torch.from_numpy(r0.copy()).cuda()
    else:
        out = torch.full((M, N), 0x7e00 if dtype == "f16" else 0x7fc0, dtype=torch.int16, device="cuda")
    K.sn_k_gemm(DT[dtype], epi, path, dev16(tiled), dev16(xb), dev16(bb) if bias else None, out, M, Wrows, Kd)
    torch.cuda.synchronize()
    if epi == K.EPI_SWIGLU16:
        g = x64 @ synth.widen(wg, dtype).T + b64[:N]
        u = x64 @ synth.widen(wu, dtype).T + b64[N:]
        want = ofw.silu(g) * u
    else:
        lin = x64 @ synth.widen(wb, dtype).T + b64
        if epi == K.EPI_GELU16:
            want = ofw.gelu(lin)
        elif epi == K.EPI_RESID32:
            want = r0.astype(np.float64) + lin
        else:
            want = lin
    got = out.cpu().numpy().astype(np.float64) if epi == K.EPI_RESID32 else synth.widen(host16(out), dtype)
    check(got, want, dtype, f"gemm path={path} epi={epi} M={M} N={N} K={Kd} bias={bias}",
          out="f32" if epi == K.EPI_RESID32 else "same")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
def test_gemm_skinny(dtype, epi):
    for i, M in enumerate([1, 8, 17, 33, 64]):
        _gemm_case(dtype, K.PATH_SKINNY, epi, M, 192, 416, bias=(i % 2 == 0), seed=10 + i)
    _gemm_case(dtype, K.PATH_SKINNY, epi, 5, 4096, 1024, bias=True, seed=20)     # 16-way K split


@pytest.mark.parametrize("epi", [0, 2, 3])
def test_gemm_skinny_wide(epi):
    """Wide weight matrices switch the decode GEMM to workgroups whose wavefronts stand side by side over
    the features and share their activation reads (2, 4 or 8 columns of wavefronts, chosen from the number
    of feature groups, the row count and the length of K); every row-tile count, ragged rows."""
    wide = 2 if epi == K.EPI_SWIGLU16 else 1
    cases = [(64, 28672, 96),       # 4 row tiles, 448 feature groups of 64: 2 columns
             (50, 51200, 64),       # 4 row tiles, 800 groups: 4 columns
             (40, 25600, 96),       # 3 row tiles, 400 groups: 2 columns
             (20, 25600, 160),      # 2 row tiles, 800 groups of 32: 4 columns
             (8, 8192, 16384),      # 1 row tile, 512 groups of 16, long K: 2 columns
             (13, 32768, 4096),     # 1 row tile, 2048 groups: 8 columns
             (32, 21504, 224)]      # 2 row tiles, 672 groups: sharing would leave the chip unevenly filled, none
    for i, (M, Nw, Kd) in enumerate(cases):
        _gemm_case("f16", K.PATH_SKINNY, epi, M, Nw // wide, Kd, bias=(i % 2 == 0), seed=70 + i)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_gemm_wide_shares_activations_through_lds(dtype):
    """9..64 token rows, row-tile packed activations and enough feature groups: the decode GEMM whose
    wavefronts fetch each activation tile once per workgroup into LDS (two k-blocks per step, double
    buffered).  Every epilogue, 1 to 4 row tiles, ragged rows, 2 and 4 column blocks per wavefront, 4 / 7 / 8
    wavefronts side by side, K ranges of odd length, K shorter than one step, K split inside the workgroup
    (from 32 k-blocks on) and across workgroups (split-K planes)."""
    cases = [(K.EPI_STORE16, 64, 32768, 96, True),        # 4 column blocks, 4 columns x 1; 3 k-blocks: odd
             (K.EPI_GELU16, 50, 28672, 160, False),       # 1792 groups of 32: 7 wavefronts side by side
             (K.EPI_SWIGLU16, 33, 16384, 32, True),       # 3 row tiles, ragged; a single k-block (shorter than a step)
             (K.EPI_SWIGLU16, 64, 28672, 1120, False),    # 35 k-blocks: split in two inside the workgroup, odd halves
             (K.EPI_STORE16, 48, 16384, 2048, True),      # 3 full row tiles, 64 k-blocks: 32 per wavefront
             (K.EPI_STORE16, 12, 32768, 96, True),        # one row tile (9..16 rows also take this kernel), ragged
             (K.EPI_GELU16, 16, 28672, 160, False),       # one full row tile, 7 wavefronts side by side
             (K.EPI_SWIGLU16, 24, 16384, 1120, True),     # two row tiles, ragged; K split inside the workgroup
             (K.EPI_STORE16, 32, 16384, 2048, False)]     # two full row tiles
    for i, (epi, M, N, Kd, bias) in enumerate(cases):
        rng = np.random.default_rng(300 + i)
        dual = epi == K.EPI_SWIGLU16
        Wrows = 2 * N if dual else N
        xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
        tiled = np.zeros(Wrows * Kd, dtype=np.uint16)
        parts = []
        for j in range(2 if dual else 1):
            wp = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.05, dtype)
            K.sn_k_tile_weights(wp, N, Kd, tiled, 2 if dual else 1, j)
            parts.append(wp)
        bb = synth.to_bits(rng.standard_normal(Wrows) * 0.3, dtype) if bias else None
        out = torch.full((M, N), 0x7e00 if dtype == "f16" else 0x7fc0, dtype=torch.int16, device="cuda")
        K.sn_k_gemm(DT[dtype], epi, K.PATH_SKINNY, dev16(tiled), dev16(K.pack_rows(xb)), dev16(bb) if bias else None, out,
                    M, Wrows, Kd, 1)
        torch.cuda.synchronize()
        x64 = synth.widen(xb, dtype)
        lin = [x64 @ synth.widen(wp, dtype).T for wp in parts]
        if bias:
            b64 = synth.widen(bb, dtype)
            lin[0] = lin[0] + b64[:N]
            if dual:
                lin[1] = lin[1] + b64[N:]
        want = ofw.silu(lin[0]) * lin[1] if dual else (ofw.gelu(lin[0]) if epi == K.EPI_GELU16 else lin[0])
        check(synth.widen(host16(out), dtype), want, dtype, f"gemm wide epi={epi} M={M} N={N} K={Kd}")
    # split-K planes (the residual projections of a 64-row decode step), packed activations
    rng = np.random.default_rng(320)
    for M, N, Kd, splits in [(64, 8192, 16384, 8), (37, 8192, 16416, 8)]:       # the second: 513 k-blocks, ragged everywhere
        xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
        wb = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.05, dtype)
        bb = synth.to_bits(rng.standard_normal(N) * 0.3, dtype)
        part = torch.full((splits, M, N), float("nan"), dtype=torch.float32, device="cuda")
        used = K.sn_k_gemm_splitk(DT[dtype], dev16(K.sn_k_tile_weights(wb, N, Kd)), dev16(K.pack_rows(xb)), dev16(bb), part,
                                  M, N, Kd, splits, 1)
        torch.cuda.synchronize()
        assert used == splits
        planes = part.cpu().numpy().astype(np.float64)
        want = synth.widen(xb, dtype) @ synth.widen(wb, dtype).T + synth.widen(bb, dtype)
        assert np.isfinite(planes).all()
        assert np.abs(planes.sum(axis=0) - want).max() <= 2e-5 * np.abs(want).max(), (M, N, Kd)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_gemm_skinny_65_to_128_rows(dtype):
    """Decode projections at 65..128 token rows: the LDS-sharing kernel with 6 or 8 row tiles where the launch
    shape allows it (packed activations, enough feature groups), two passes of up to 64 rows otherwise (few
    feature groups, or row-major activations); every epilogue; split-K planes on both paths."""
    cases = [(K.EPI_STORE16, 65, 16384, 96, True, True),      # 6 row tiles, 5 of them real
             (K.EPI_SWIGLU16, 96, 16384, 160, False, True),
             (K.EPI_GELU16, 128, 28672, 1056, True, True),    # 8 row tiles, 7 wavefronts side by side, odd k-block count
             (K.EPI_STORE16, 100, 192, 416, True, True),      # few feature groups: two passes, packed
             (K.EPI_SWIGLU16, 128, 320, 96, False, False),    # two passes, row-major
             (K.EPI_RESID32, 77, 192, 416, True, False)]
    for i, (epi, M, N, Kd, bias, packed) in enumerate(cases):
        rng = np.random.default_rng(400 + i)
        dual = epi == K.EPI_SWIGLU16
        Wrows = 2 * N if dual else N
        xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
        tiled = np.zeros(Wrows * Kd, dtype=np.uint16)
        parts = []
        for j in range(2 if dual else 1):
            wp = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.05, dtype)
            K.sn_k_tile_weights(wp, N, Kd, tiled, 2 if dual else 1, j)
            parts.append(wp)
        bb = synth.to_bits(rng.standard_normal(Wrows) * 0.3, dtype) if bias else None
        x64 = synth.widen(xb, dtype)
        lin = [x64 @ synth.widen(wp, dtype).T for wp in parts]
        if bias:
            b64 = synth.widen(bb, dtype)
            lin[0] = lin[0] + b64[:N]
            if dual:
                lin[1] = lin[1] + b64[N:]
        xdev = dev16(K.pack_rows(xb) if packed else xb)
        if epi == K.EPI_RESID32:
            r0 = rng.standard_normal((M, N)).astype(np.float32)
            out = torch.from_numpy(r0.copy()).cuda()
            want = r0.astype(np.float64) + lin[0]
        else:
            out = torch.full((M, N), 0x7e00 if dtype == "f16" else 0x7fc0, dtype=torch.int16, device="cuda")
            want = ofw.silu(lin[0]) * lin[1] if dual else (ofw.gelu(lin[0]) if epi == K.EPI_GELU16 else lin[0])
        K.sn_k_gemm(DT[dtype], epi, K.PATH_SKINNY, dev16(tiled), xdev, dev16(bb) if bias else None, out, M, Wrows, Kd,
                    1 if packed else 0)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64) if epi == K.EPI_RESID32 else synth.widen(host16(out), dtype)
        check(got, want, dtype, f"gemm {M} rows epi={epi} N={N} K={Kd} packed={packed}", out="f32" if epi == K.EPI_RESID32 else "same")
    rng = np.random.default_rng(420)
    for M, N, Kd, splits, packed in [(128, 8192, 16384, 8, True), (70, 256, 1024, 3, True), (90, 192, 416, 2, False)]:
        xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
        wb = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.05, dtype)
        bb = synth.to_bits(rng.standard_normal(N) * 0.3, dtype)
        part = torch.full((splits, M, N), float("nan"), dtype=torch.float32, device="cuda")
        used = K.sn_k_gemm_splitk(DT[dtype], dev16(K.sn_k_tile_weights(wb, N, Kd)), dev16(K.pack_rows(xb) if packed else xb), dev16(bb),
                                  part, M, N, Kd, splits, 1 if packed else 0)
        torch.cuda.synchronize()
        assert used == splits
        planes = part.cpu().numpy().astype(np.float64)
        want = synth.widen(xb, dtype) @ synth.widen(wb, dtype).T + synth.widen(bb, dtype)
        assert np.isfinite(planes).all(), (M, N, Kd)
        assert np.abs(planes.sum(axis=0) - want).max() <= 2e-5 * np.abs(want).max(), (M, N, Kd)


@pytest.mark.parametrize("case", ["c2_ffn_up", "c3_ffn_up", "c5_qkv", "c5_ffn_up"])
def test_gemm_skinny_full_size_sampled(case):
    """Decode projections at the benchmark workloads' real shapes and row counts, in the launch configuration a
    decode step uses (row-tile packed activations in): sampled output features against the oracle's arithmetic
    (float64 products of the same 16-bit inputs), all rows."""
    M, Wrows, Kd, epi, bias = {"c2_ffn_up": (8, 16384, 4096, K.EPI_GELU16, True),
                               "c3_ffn_up": (32, 27648, 5120, K.EPI_SWIGLU16, False),
                               "c5_qkv": (64, 10240, 8192, K.EPI_STORE16, False),
                               "c5_ffn_up": (64, 57344, 8192, K.EPI_SWIGLU16, False)}[case]
    rng = np.random.default_rng(90)
    dual = epi == K.EPI_SWIGLU16
    N = Wrows // 2 if dual else Wrows
    xb = synth.to_bits(rng.standard_normal((M, Kd)), "f16")
    tiled = np.zeros(Wrows * Kd, dtype=np.uint16)
    parts = []
    for i in range(2 if dual else 1):
        wpart = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.02, "f16")
        K.sn_k_tile_weights(wpart, N, Kd, tiled, 2 if dual else 1, i)
        parts.append(wpart)
    bb = synth.to_bits(rng.standard_normal(Wrows) * 0.3, "f16") if bias else None
    out = torch.full((M, N), 0x7e00, dtype=torch.int16, device="cuda")
    K.sn_k_gemm(DT["f16"], epi, K.PATH_SKINNY, dev16(tiled), dev16(K.pack_rows(xb)), dev16(bb) if bias else None, out,
                M, Wrows, Kd, 1)
    torch.cuda.synchronize()
    cols = np.unique(np.concatenate([[0, 1, 15, 16, 63, 64, N - 65, N - 1], rng.integers(0, N, 400)]))
    x64 = synth.widen(xb, "f16")
    lin = [x64 @ synth.widen(wp[cols], "f16").T for wp in parts]
    if bias:
        lin[0] = lin[0] + synth.widen(bb, "f16")[cols]
    want = ofw.silu(lin[0]) * lin[1] if dual else (ofw.gelu(lin[0]) if epi == K.EPI_GELU16 else lin[0])
    got = synth.widen(host16(out), "f16")
    assert np.isfinite(got).all()
    check(got[:, cols], want, "f16", f"gemm_skinny full size {case}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
def test_gemm_tile(dtype, epi):
    for i, M in enumerate([1, 127, 300]):
        _gemm_case(dtype, K.PATH_TILE, epi, M, 192, 416, bias=(i % 2 == 0), seed=30 + i)
    _gemm_case(dtype, K.PATH_TILE, epi, 130, 384, 64, bias=True, seed=40)


@pytest.mark.parametrize("dtype,epi", [("f16", 0), ("f16", 1), ("bf16", 2), ("bf16", 3), ("f16", 3)])
def test_gemm_tile_large_m(dtype, epi):
    """With more than 128 rows (and N, K multiples of 256) the prefill GEMM uses its 256-token x 256-feature
    workgroup tile: direct-to-LDS activation loads, an 8-deep operand ring (one, two and three trips of the
    unrolled k loop), outputs transposed through LDS, a ragged last token tile, the XCD-banded numbering
    (32 feature tiles) and the plain one (33); a single round of few tiles (300 rows); the smallest row counts it takes (129: one
    token tile with 127 idle rows; 257: a second tile for one row).  The last case, K = 224, stays with the 128 x 256 kernel."""
    wide = 2 if epi == K.EPI_SWIGLU16 else 1      # SwiGLU: N counts output features, the weight has 2 N rows
    for i, (M, Nw, Kd) in enumerate([(12400, 8192, 256), (12300, 8448, 512), (12481, 8192, 768), (300, 1024, 512), (129, 512, 256), (257, 256, 512),
                                      (1250, 256, 224)]):
        _gemm_case(dtype, K.PATH_TILE, epi, M, Nw // wide, Kd, bias=(i % 2 == 0), seed=50 + i)


@pytest.mark.parametrize("epi", [0, 2, 3])
def test_gemm_tile_large_m_packed_activations(epi):
    """The 256 x 256 prefill GEMM reading row-tile packed activations (one contiguous KiB per 16-token x 32-k tile,
    whole cache lines per request): the layout is a permutation of the operand fetch only, so the output must equal,
    bit for bit, that of the same launch on the row-major matrix -- which test_gemm_tile_large_m checks against the
    oracle.  Ragged last token tile; shapes the smaller kernels would take refuse the flag."""
    rng = np.random.default_rng(77)
    wide = 2 if epi == K.EPI_SWIGLU16 else 1
    M, N, Kd = 12481, 8192 // wide, 512
    xb = synth.to_bits(rng.standard_normal((M, Kd)), "f16")
    tiled = np.zeros(N * wide * Kd, dtype=np.uint16)
    for j in range(wide):
        K.sn_k_tile_weights(synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.05, "f16"), N, Kd, tiled, wide, j)
    outs = []
    for flags, xdev in ((0, dev16(xb)), (1, dev16(K.pack_rows(xb)))):
        if epi == K.EPI_RESID32:
            out = torch.ones(M, N, dtype=torch.float32, device="cuda")
        else:
            out = torch.full((M, N), 0x7e00, dtype=torch.int16, device="cuda")
        K.sn_k_gemm(DT["f16"], epi, K.PATH_TILE, dev16(tiled), xdev, None, out, M, N * wide, Kd, flags)
        torch.cuda.synchronize()
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
    assert bool(torch.isfinite(outs[1].float()).all()) if epi == K.EPI_RESID32 else bool((outs[1] != 0x7e00).any())
    if epi != K.EPI_RESID32:            # the 16-bit output written row-tile packed as well (it feeds the next projection)
        Mp = (M + 15) // 16 * 16
        outp = torch.zeros(Mp * N, dtype=torch.int16, device="cuda")
        K.sn_k_gemm(DT["f16"], epi, K.PATH_TILE, dev16(tiled), dev16(K.pack_rows(xb)), None, outp, M, N * wide, Kd, 3)
        torch.cuda.synchronize()
        assert np.array_equal(K.unpack_rows(host16(outp), M, N), host16(outs[0]))
    with pytest.raises(sn.SnError):     # 128 x 256 kernel (at most 128 rows): row-major only
        K.sn_k_gemm(DT["f16"], epi, K.PATH_TILE, dev16(tiled), dev16(K.pack_rows(xb[:112])), None, outs[1], 112, N * wide, Kd, 1)


def _kv_setup(rng, dtype, lens_before, n_new, caps, Hq, Hkv, d, rope):
    """Random qkv rows for the new tokens and a random cache prefix; returns device index
    arrays, device buffers and float64 views for the oracle."""
    B = len(caps)
    T = sum(n_new)
    qkv = synth.to_bits(rng.standard_normal((T, (Hq + 2 * Hkv) * d)), dtype)
    kv_off = np.concatenate([[0], np.cumsum(caps)[:-1]]).astype(np.int32)
    kv = np.zeros(int(sum(caps)) * 2 * Hkv * d, dtype=np.uint16)
    Kc, Vc = [], []
    for b in range(B):
        kb = synth.to_bits(rng.standard_normal((lens_before[b], Hkv, d)), dtype)
        vb = synth.to_bits(rng.standard_normal((lens_before[b], Hkv, d)), dtype)
        Kc.append(kb)
        Vc.append(vb)
        base = int(kv_off[b]) * 2 * Hkv * d
        blk = kv[base: base + caps[b] * 2 * Hkv * d].reshape(Hkv, 2, caps[b], d)
        blk[:, 0, :lens_before[b]] = kb.transpose(1, 0, 2)
        blk[:, 1, :lens_before[b]] = vb.transpose(1, 0, 2)
    tok_seq = np.concatenate([[b] * n_new[b] for b in range(B)]).astype(np.int32)
    tok_pos = np.concatenate([np.arange(lens_before[b], lens_before[b] + n_new[b]) for b in range(B)]).astype(np.int32)
    tok_start = np.concatenate([[0], np.cumsum(n_new)[:-1]]).astype(np.int32)
    inv_freq = (10000.0 ** (-2.0 * np.arange(d // 2) / d)).astype(np.float32)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    dev = dict(qkv=dev16(qkv), kv=dev16(kv), tok_seq=i32(tok_seq), tok_pos=i32(tok_pos), kv_off=i32(kv_off),
               cap=i32(caps), len_before=i32(lens_before), n_new=i32(n_new), tok_start=i32(tok_start),
               inv_freq=torch.from_numpy(inv_freq).cuda())
    return qkv, Kc, Vc, kv_off, tok_start, dev


def _oracle_attention(dtype, qkv, Kc, Vc, lens_before, n_new, tok_start, Hq, Hkv, d, rope):
    outs, k_new, v_new, q_rot = [], [], [], []
    for b in range(len(n_new)):
        rows = synth.widen(qkv[tok_start[b]: tok_start[b] + n_new[b]], dtype)
        q = rows[:, :Hq * d].reshape(-1, Hq, d)
        k = rows[:, Hq * d:(Hq + Hkv) * d].reshape(-1, Hkv, d)
        v = rows[:, (Hq + Hkv) * d:].reshape(-1, Hkv, d)
        pos = np.arange(lens_before[b], lens_before[b] + n_new[b])
        if rope:
            q = ofw.rope(q, pos[:, None], 10000.0)
            k = ofw.rope(k, pos[:, None], 10000.0)
        k = ofw.round_to_storage(k, dtype)
        v = ofw.round_to_storage(v, dtype)
        Kf = np.concatenate([synth.widen(Kc[b], dtype), k], axis=0)
        Vf = np.concatenate([synth.widen(Vc[b], dtype), v], axis=0)
        outs.append(ofw.causal_attention(q, Kf, Vf, lens_before[b]).reshape(n_new[b], Hq * d))
        k_new.append(k)
        v_new.append(v)
        q_rot.append(q)
    return np.concatenate(outs, axis=0), k_new, v_new, q_rot


@pytest.mark.parametrize("dtype,Hq,Hkv,d,rope", [("f16", 4, 4, 64, False), ("bf16", 8, 8, 128, True),
                                                 ("bf16", 16, 2, 128, True), ("f16", 6, 3, 64, True),
                                                 ("f16", 8, 2, 128, True), ("f16", 16, 2, 128, False),
                                                 ("f16", 8, 2, 64, True)])
def test_rope_append_and_attn_decode(dtype, Hq, Hkv, d, rope):
    rng = np.random.default_rng(3)
    lens_before = [0, 1, 130, 517, 63]
    B = len(lens_before)
    caps = [l + 3 for l in lens_before]
    n_new = [1] * B
    qkv, Kc, Vc, kv_off, tok_start, dv = _kv_setup(rng, dtype, lens_before, n_new, caps, Hq, Hkv, d, rope)
    mirror = torch.zeros_like(dv["kv"])
    K.sn_k_rope_append(DT[dtype], DT[dtype], dv["qkv"], dv["tok_seq"], dv["tok_pos"], dv["kv_off"], dv["cap"], dv["kv"], mirror,
                       dv["inv_freq"], B, Hq, Hkv, d, rope)
    want, k_new, v_new, q_rot = _oracle_attention(dtype, qkv, Kc, Vc, lens_before, n_new, tok_start, Hq, Hkv, d, rope)
    torch.cuda.synchronize()
    kv_host = host16(dv["kv"])
    mir_host = host16(mirror)
    for b in range(B):
        base = int(kv_off[b]) * 2 * Hkv * d
        blk = kv_host[base: base + caps[b] * 2 * Hkv * d].reshape(Hkv, 2, caps[b], d)
        mblk = mir_host[base: base + caps[b] * 2 * Hkv * d].reshape(Hkv, 2, caps[b], d)
        p = lens_before[b]
        check(synth.widen(blk[:, 0, p], dtype), k_new[b][0], dtype, f"appended k seq {b}", want_is_rounded=True)
        assert np.array_equal(synth.widen(blk[:, 1, p], dtype), v_new[b][0])          # v is copied bit for bit
        assert np.array_equal(blk[:, :, p], mblk[:, :, p])                              # mirror gets the same rows
        assert np.array_equal(blk[:, 0, :p], Kc[b].transpose(1, 0, 2))                  # the prefix is untouched
        assert not mblk[:, :, :p].any() and not mblk[:, :, p + 1:].any()
    q_got = synth.widen(host16(dv["qkv"]), dtype)[:, :Hq * d].reshape(B, Hq, d)
    check(q_got, np.concatenate(q_rot, axis=0), dtype, "rotated q")
    for S in (0, 1, 3, 16):
        out = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
        part = torch.zeros(B * Hq * 16 * (d + 2), dtype=torch.float32, device="cuda")
        K.sn_k_attn_decode(DT[dtype], dv["qkv"], dv["kv"], dv["len_before"], dv["kv_off"], dv["cap"], out, part, B, Hq,
                           Hkv, d, S, max(lens_before) + 1)
        torch.cuda.synchronize()
        check(synth.widen(host16(out), dtype), want, dtype, f"attn_decode S={S}", per_row=True, bar=C_ATTN[dtype])


@pytest.mark.parametrize("dtype,Hq,Hkv,d,rope", [("f16", 4, 4, 64, False), ("bf16", 8, 8, 128, True),
                                                 ("bf16", 16, 2, 128, True), ("f16", 6, 3, 64, True),
                                                 ("f16", 8, 2, 64, True), ("f16", 32, 32, 128, False),
                                                 ("f16", 8, 2, 128, True), ("f16", 16, 2, 128, False)])
def test_attn_decode_with_fused_append(dtype, Hq, Hkv, d, rope):
    """The decode kernel that rotates, appends and attends in one launch: against the oracle,
    and bit for bit against rope_append followed by attn_decode (outputs, cache rows, mirror);
    the QKV buffer must be left as it was."""
    rng = np.random.default_rng(13)
    lens_before = [0, 1, 130, 517, 63, 31, 32]
    B = len(lens_before)
    caps = [l + 2 for l in lens_before]
    n_new = [1] * B
    qkv, Kc, Vc, kv_off, tok_start, dv = _kv_setup(rng, dtype, lens_before, n_new, caps, Hq, Hkv, d, rope)
    want, k_new, v_new, _ = _oracle_attention(dtype, qkv, Kc, Vc, lens_before, n_new, tok_start, Hq, Hkv, d, rope)
    kv0 = dv["kv"].clone()
    qkv0 = dv["qkv"].clone()
    part = torch.zeros(B * Hq * 16 * (d + 2), dtype=torch.float32, device="cuda")
    # reference pair of kernels on its own copies
    kv_two, qkv_two, mir_two = kv0.clone(), qkv0.clone(), torch.zeros_like(kv0)
    K.sn_k_rope_append(DT[dtype], DT[dtype], qkv_two, dv["tok_seq"], dv["tok_pos"], dv["kv_off"], dv["cap"], kv_two, mir_two,
                       dv["inv_freq"], B, Hq, Hkv, d, rope)
    for S in (0, 1, 3, 16):
        out_two = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
        K.sn_k_attn_decode(DT[dtype], qkv_two, kv_two, dv["len_before"], dv["kv_off"], dv["cap"], out_two, part, B, Hq,
                           Hkv, d, S, max(lens_before) + 1)
        kv_f, mir_f = kv0.clone(), torch.zeros_like(kv0)
        out_f = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
        K.sn_k_attn_decode_append(DT[dtype], dv["qkv"], kv_f, mir_f, dv["inv_freq"], rope, dv["len_before"], dv["kv_off"],
                                  dv["cap"], out_f, part, B, Hq, Hkv, d, S, max(lens_before) + 1)
        torch.cuda.synchronize()
        check(synth.widen(host16(out_f), dtype), want, dtype, f"fused attn_decode S={S}", per_row=True, bar=C_ATTN[dtype])
        assert torch.equal(dv["qkv"], qkv0), "the fused kernel must not modify the QKV buffer"
        assert torch.equal(kv_f, kv_two), f"cache after the fused kernel differs from rope_append's (S={S})"
        assert torch.equal(mir_f, mir_two), f"mirror differs (S={S})"
        assert torch.equal(out_f, out_two), f"fused output differs from the two-kernel path (S={S})"
        # the same step with q, k, v handed over as split-K partial planes (what a 9..128-row decode step
        # does): three planes that add up, in fp32 and in this order, to exactly the 16-bit values -- so
        # the result must not differ in a single bit; rows and planes the kernel must not read hold NaN
        q32 = torch.from_numpy(synth.widen(host16(qkv0), dtype).astype(np.float32)).cuda().reshape(B, -1)
        planes = torch.full((5, B + 3, q32.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
        planes[0, :B], planes[1, :B], planes[2, :B] = 0.5 * q32, 0.25 * q32, 0.25 * q32
        kv_p, mir_p = kv0.clone(), torch.zeros_like(kv0)
        out_p = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
        K.sn_k_attn_decode_append_planes(DT[dtype], planes, 3, B + 3, kv_p, mir_p, dv["inv_freq"], rope, dv["len_before"],
                                         dv["kv_off"], dv["cap"], out_p, part, B, Hq, Hkv, d, S, max(lens_before) + 1)
        torch.cuda.synchronize()
        assert torch.equal(out_p, out_f) and torch.equal(kv_p, kv_f) and torch.equal(mir_p, mir_f), f"planes path differs (S={S})"
    kv_host = host16(kv_f)
    for b in range(B):
        base = int(kv_off[b]) * 2 * Hkv * d
        blk = kv_host[base: base + caps[b] * 2 * Hkv * d].reshape(Hkv, 2, caps[b], d)
        p = lens_before[b]
        check(synth.widen(blk[:, 0, p], dtype), k_new[b][0], dtype, f"appended k seq {b}", want_is_rounded=True)
        assert np.array_equal(synth.widen(blk[:, 1, p], dtype), v_new[b][0])


@pytest.mark.parametrize("dtype,Hq,Hkv,d,rope", [("f16", 4, 4, 64, False), ("bf16", 8, 8, 128, True),
                                                 ("bf16", 8, 2, 128, True), ("f16", 8, 2, 128, True),
                                                 ("f16", 4, 4, 128, False), ("bf16", 4, 2, 64, True),
                                                 ("f16", 6, 2, 128, True)])   # 36 work items: not a multiple of the 8 XCDs
def test_attn_prefill(dtype, Hq, Hkv, d, rope):
    rng = np.random.default_rng(4)
    lens_before = [0, 0, 40, 0]
    n_new = [1, 128, 37, 300]         # single token, exact tile, chunk on top of a cached prefix, ragged multi-tile
    B = len(n_new)
    caps = [lens_before[b] + n_new[b] + 2 for b in range(B)]
    qkv, Kc, Vc, kv_off, tok_start, dv = _kv_setup(rng, dtype, lens_before, n_new, caps, Hq, Hkv, d, rope)
    T = sum(n_new)
    K.sn_k_rope_append(DT[dtype], DT[dtype], dv["qkv"], dv["tok_seq"], dv["tok_pos"], dv["kv_off"], dv["cap"], dv["kv"], None,
                       dv["inv_freq"], T, Hq, Hkv, d, rope)
    tile_seq, tile_q0 = [], []
    for b in range(B):
        for q0 in range(0, n_new[b], K.SN_K_PREFILL_QTILE):
            tile_seq.append(b)
            tile_q0.append(q0)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    out = torch.zeros(T, Hq * d, dtype=torch.int16, device="cuda")
    K.sn_k_attn_prefill(DT[dtype], dv["qkv"], dv["kv"], dv["len_before"], dv["n_new"], dv["tok_start"], dv["kv_off"],
                        dv["cap"], i32(tile_seq), i32(tile_q0), out, len(tile_seq), Hq, Hkv, d)
    torch.cuda.synchronize()
    want, *_ = _oracle_attention(dtype, qkv, Kc, Vc, lens_before, n_new, tok_start, Hq, Hkv, d, rope)
    check(synth.widen(host16(out), dtype), want, dtype, "attn_prefill", per_row=True, bar=C_ATTN[dtype])
    # the same launch writing its output row-tile packed (what feeds a packed output projection)
    outp = torch.zeros((T + 15) // 16 * 16 * Hq * d, dtype=torch.int16, device="cuda")
    K.sn_k_attn_prefill(DT[dtype], dv["qkv"], dv["kv"], dv["len_before"], dv["n_new"], dv["tok_start"], dv["kv_off"],
                        dv["cap"], i32(tile_seq), i32(tile_q0), outp, len(tile_seq), Hq, Hkv, d, 1)
    torch.cuda.synchronize()
    assert np.array_equal(K.unpack_rows(host16(outp), T, Hq * d), host16(out))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_casts_are_exact(dtype):
    rng = np.random.default_rng(5)
    bits = synth.to_bits(rng.standard_normal(5000) * 4, dtype)
    x = torch.zeros(5000, dtype=torch.float32, device="cuda")
    K.sn_k_cast_in(DT[dtype], dev16(bits), x, 5000)
    back = torch.zeros(5000, dtype=torch.int16, device="cuda")
    K.sn_k_cast_out(DT[dtype], x, back, 5000)
    torch.cuda.synchronize()
    assert np.array_equal(x.cpu().numpy().astype(np.float64), synth.widen(bits, dtype))
    assert np.array_equal(host16(back), bits)
    # rounding fp32 -> 16 bit is nearest-even, as the oracle's storage rounding
    f = (rng.standard_normal(5000) * 4).astype(np.float32)
    K.sn_k_cast_out(DT[dtype], torch.from_numpy(f).cuda(), back, 5000)
    torch.cuda.synchronize()
    assert np.array_equal(synth.widen(host16(back), dtype), ofw.round_to_storage(f.astype(np.float64), dtype))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("splits", [0, 1, 3, 8])
def test_splitk_projection_folded_into_norm_and_cast(dtype, splits):
    """Residual projection as split-K partials, folded into the residual stream by the next
    norm (and by the final cast): x + bias + X W^T, then LayerNorm / 16-bit rounding."""
    rng = np.random.default_rng(6)
    for M, N, Kd in [(8, 256, 1024), (33, 192, 416), (64, 512, 2048)]:
        xb = synth.to_bits(rng.standard_normal((M, Kd)), dtype)
        wb = synth.to_bits(rng.standard_normal((N, Kd)) * 0.05, dtype)
        bb = synth.to_bits(rng.standard_normal(N) * 0.3, dtype)
        g = synth.to_bits(1 + 0.1 * rng.standard_normal(N), dtype)
        sh = synth.to_bits(0.1 * rng.standard_normal(N), dtype)
        r0 = rng.standard_normal((M, N)).astype(np.float32)
        tiled = K.sn_k_tile_weights(wb, N, Kd)
        part = torch.full((8, M, N), float("nan"), dtype=torch.float32, device="cuda")
        # the bias may be added by the projection itself (plane 0; what an iteration does) or by the fold
        bias_in_gemm = (M != 33)
        used = K.sn_k_gemm_splitk(DT[dtype], dev16(tiled), dev16(xb), dev16(bb) if bias_in_gemm else None, part,
                                  M, N, Kd, splits)
        fold_bias = None if bias_in_gemm else dev16(bb)
        assert used == splits or (splits == 0 and 1 <= used <= 8)
        want_x = r0.astype(np.float64) + synth.widen(bb, dtype) + synth.widen(xb, dtype) @ synth.widen(wb, dtype).T
        # folded into a LayerNorm
        x = torch.from_numpy(r0.copy()).cuda()
        out = torch.zeros(M, N, dtype=torch.int16, device="cuda")
        K.sn_k_norm_fold(DT[dtype], True, x, dev16(g), dev16(sh), out, M, N, 1e-5, part, used, fold_bias, 0)
        torch.cuda.synchronize()
        got_x = x.cpu().numpy().astype(np.float64)
        assert np.abs(got_x - want_x).max() <= 2e-5 * np.abs(want_x).max(), (M, N, Kd)
        want_u = ofw.layer_norm(want_x, synth.widen(g, dtype), synth.widen(sh, dtype), 1e-5)
        check(synth.widen(host16(out), dtype), want_u, dtype, f"norm_fold M={M} N={N} K={Kd} splits={used}")
        # folded into the final cast
        x2 = torch.from_numpy(r0.copy()).cuda()
        K.sn_k_cast_out_fold(DT[dtype], x2, out, M, N, part, used, fold_bias)
        torch.cuda.synchronize()
        assert np.array_equal(x2.cpu().numpy(), x.cpu().numpy())               # same fixed-order sum
        assert np.array_equal(synth.widen(host16(out), dtype), ofw.round_to_storage(got_x, dtype))


def test_splitk_projection_wide_and_long():
    """3-4 row tiles, at least 800 feature groups of 64 per 8 splits and a long K per split: the split-K
    projection runs 4 columns of 2 wavefronts that share their activation reads; planes must add up to
    X W^T + bias, with the bias in plane 0 only."""
    rng = np.random.default_rng(8)
    # the last case: one row tile and 256 feature groups -- the library picks no split at all (8 wavefronts split K)
    for M, N, Kd, splits in [(64, 8192, 16384, 8), (40, 12800, 8192, 4), (8, 4096, 16384, 0)]:
        xb = synth.to_bits(rng.standard_normal((M, Kd)), "f16")
        wb = synth.to_bits(rng.standard_normal((N, Kd)) * 0.05, "f16")
        bb = synth.to_bits(rng.standard_normal(N) * 0.3, "f16")
        tiled = K.sn_k_tile_weights(wb, N, Kd)
        part = torch.full((max(splits, 8), M, N), float("nan"), dtype=torch.float32, device="cuda")
        used = K.sn_k_gemm_splitk(DT["f16"], dev16(tiled), dev16(xb), dev16(bb), part, M, N, Kd, splits)
        torch.cuda.synchronize()
        assert used == (splits if splits else 1)
        planes = part[:used].cpu().numpy().astype(np.float64)
        want = synth.widen(xb, "f16") @ synth.widen(wb, "f16").T + synth.widen(bb, "f16")
        got = planes.sum(axis=0)
        assert np.isfinite(planes).all()
        assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max(), (M, N, Kd)
        # plane s holds the s-th K range only: plane 1 equals that range's product, without the bias
        if used > 1:
            kr = Kd // used
            want1 = synth.widen(xb, "f16")[:, kr:2 * kr] @ synth.widen(wb, "f16")[:, kr:2 * kr].T
            assert np.abs(planes[1] - want1).max() <= 2e-5 * np.abs(want).max()


@pytest.mark.parametrize("case", ["c5_qkv", "c5_oproj", "c5_ffn_down", "c4_qkv", "c3_ffn_down", "c3_qkv", "c4_qkv_12"])
def test_splitk_projection_planned_shapes_full_size(case):
    """Split-K projections at the real shapes and row counts of the 13B-, 30B- and 70B-shaped decode steps, with
    the number of planes and the launch shape the library plans itself (packed activations in, as in a decode
    step): the planes add up to X W^T + bias on sampled features, all rows."""
    M, N, Kd = {"c5_qkv": (64, 10240, 8192), "c5_oproj": (64, 8192, 8192), "c5_ffn_down": (64, 8192, 28672),
                "c4_qkv": (64, 21504, 7168), "c3_ffn_down": (32, 5120, 13824), "c3_qkv": (32, 15360, 5120),
                "c4_qkv_12": (12, 21504, 7168)}[case]
    rng = np.random.default_rng(91)
    xb = synth.to_bits(rng.standard_normal((M, Kd)), "f16")
    wb = synth.to_bits(rng.standard_normal((N, Kd), dtype=np.float32) * 0.02, "f16")
    bb = synth.to_bits(rng.standard_normal(N) * 0.3, "f16")
    part = torch.full((8, M, N), float("nan"), dtype=torch.float32, device="cuda")
    used = K.sn_k_gemm_splitk(DT["f16"], dev16(K.sn_k_tile_weights(wb, N, Kd)), dev16(K.pack_rows(xb)), dev16(bb), part,
                              M, N, Kd, 0, 1)
    torch.cuda.synchronize()
    assert 2 <= used <= 8, used
    planes = part[:used].cpu().numpy().astype(np.float64)
    assert np.isfinite(planes).all() and bool(torch.isnan(part[used:]).all())
    cols = np.unique(np.concatenate([[0, 1, 15, 16, 63, 64, N - 65, N - 1], rng.integers(0, N, 400)]))
    want = synth.widen(xb, "f16") @ synth.widen(wb[cols], "f16").T + synth.widen(bb, "f16")[cols]
    got = planes.sum(axis=0)[:, cols]
    assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max() + 1e-6, case
    # every plane carries a share: a launch shape that dropped a K range would leave one at zero
    assert all(np.abs(planes[i]).max() > 0 for i in range(used))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_packed_activation_layout_through_norm_gemm_and_attention(dtype):
    """The row-tile packed layout is only a permutation: every kernel that can read or write
    it must produce exactly the bits of its row-major form."""
    rng = np.random.default_rng(7)
    for M in (1, 8, 17, 64):
        h, N = 416, 192
        Mp = (M + 15) // 16 * 16
        x = (rng.standard_normal((M, h)) * 2).astype(np.float32)
        g = synth.to_bits(1 + 0.1 * rng.standard_normal(h), dtype)
        sh = synth.to_bits(0.1 * rng.standard_normal(h), dtype)
        u_row = torch.zeros(M, h, dtype=torch.int16, device="cuda")
        u_pk = torch.zeros(Mp * h, dtype=torch.int16, device="cuda")
        xd = torch.from_numpy(x).cuda()
        K.sn_k_norm_fold(DT[dtype], True, xd, dev16(g), dev16(sh), u_row, M, h, 1e-5, None, 0, None, 0)
        K.sn_k_norm_fold(DT[dtype], True, xd, dev16(g), dev16(sh), u_pk, M, h, 1e-5, None, 0, None, 1)
        torch.cuda.synchronize()
        u = host16(u_row)
        assert np.array_equal(K.unpack_rows(host16(u_pk), M, h), u)
        assert np.array_equal(K.pack_rows(u)[K.sn_k_packed_offset(M - 1, h - 1, h)], u[M - 1, h - 1])
        wb = synth.to_bits(rng.standard_normal((N, h)) * 0.05, dtype)
        tiled = dev16(K.sn_k_tile_weights(wb, N, h))
        for epi in (K.EPI_STORE16, K.EPI_GELU16):
            ref = torch.zeros(M, N, dtype=torch.int16, device="cuda")
            K.sn_k_gemm(DT[dtype], epi, K.PATH_SKINNY, tiled, u_row, None, ref, M, N, h, 0)
            a = torch.zeros(M, N, dtype=torch.int16, device="cuda")
            K.sn_k_gemm(DT[dtype], epi, K.PATH_SKINNY, tiled, u_pk, None, a, M, N, h, 1)            # packed in
            b = torch.zeros(Mp * N, dtype=torch.int16, device="cuda")
            K.sn_k_gemm(DT[dtype], epi, K.PATH_SKINNY, tiled, u_pk, None, b, M, N, h, 3)            # packed in and out
            torch.cuda.synchronize()
            assert np.array_equal(host16(a), host16(ref))
            assert np.array_equal(K.unpack_rows(host16(b), M, N), host16(ref))
    # many rows (a prefill's norm): the packed writer walks the rows tile by tile within an XCD; ragged row count
    for M, h in ((1000, 416), (2051, 1024)):
        x = (rng.standard_normal((M, h)) * 2).astype(np.float32)
        g = synth.to_bits(1 + 0.1 * rng.standard_normal(h), dtype)
        u_row = torch.zeros(M, h, dtype=torch.int16, device="cuda")
        u_pk = torch.full(((M + 15) // 16 * 16 * h,), 0x7e00, dtype=torch.int16, device="cuda")
        xd = torch.from_numpy(x).cuda()
        K.sn_k_norm_fold(DT[dtype], False, xd, dev16(g), None, u_row, M, h, 1e-5, None, 0, None, 0)
        K.sn_k_norm_fold(DT[dtype], False, xd, dev16(g), None, u_pk, M, h, 1e-5, None, 0, None, 1)
        torch.cuda.synchronize()
        assert np.array_equal(K.unpack_rows(host16(u_pk), M, h), host16(u_row))
        assert np.array_equal(xd.cpu().numpy(), x)                    # no fold: the fp32 rows are left alone
    # decode attention writing packed output
    Hq, Hkv, d = 8, 2, 128
    lens_before = [5, 300, 0]
    B = len(lens_before)
    caps = [l + 2 for l in lens_before]
    qkv, Kc, Vc, kv_off, tok_start, dv = _kv_setup(rng, dtype, lens_before, [1] * B, caps, Hq, Hkv, d, True)
    K.sn_k_rope_append(DT[dtype], DT[dtype], dv["qkv"], dv["tok_seq"], dv["tok_pos"], dv["kv_off"], dv["cap"], dv["kv"], None,
                       dv["inv_freq"], B, Hq, Hkv, d, True)
    part = torch.zeros(B * Hq * 16 * (d + 2), dtype=torch.float32, device="cuda")
    for S in (1, 2):
        ref = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
        pk = torch.zeros(16 * Hq * d, dtype=torch.int16, device="cuda")
        K.sn_k_attn_decode(DT[dtype], dv["qkv"], dv["kv"], dv["len_before"], dv["kv_off"], dv["cap"], ref, part, B, Hq, Hkv, d, S, 301, 0)
        K.sn_k_attn_decode(DT[dtype], dv["qkv"], dv["kv"], dv["len_before"], dv["kv_off"], dv["cap"], pk, part, B, Hq, Hkv, d, S, 301, 1)
        torch.cuda.synchronize()
        assert np.array_equal(K.unpack_rows(host16(pk), B, Hq * d), host16(ref))
