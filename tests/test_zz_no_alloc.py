"""The entry point for callers that cannot allocate (sn_k_attn_decode_static): decode attention whose
key-range partials live in the library's own static device buffer.  Its output must equal, bit for bit,
that of sn_k_attn_decode with a caller-supplied buffer -- on two calls in a row, the second on a smaller
input (the buffer keeps the first call's contents) -- and match the CPU oracle; free device memory must
not move across a call; a request beyond the buffer is refused with a message."""
import numpy as np
import pytest
import torch

from oracle import forward as ofw
from paper_2502_08182_amd import sn, synth
from paper_2502_08182_amd import sn_kernels as K

pytestmark = pytest.mark.gpu


def _dev16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _case(seed, lens_before, Hq, Hkv, d):
    """Random rotated queries and a cache that already holds the step's own row; returns device
    buffers and the oracle's attention output (float64)."""
    rng = np.random.default_rng(seed)
    B = len(lens_before)
    caps = [l + 1 for l in lens_before]
    kv_off = np.concatenate([[0], np.cumsum(caps)[:-1]]).astype(np.int32)
    qkv = synth.to_bits(rng.standard_normal((B, (Hq + 2 * Hkv) * d)), "f16")
    kv = np.zeros(int(sum(caps)) * 2 * Hkv * d, dtype=np.uint16)
    want = []
    for b in range(B):
        n = caps[b]
        kb = synth.to_bits(rng.standard_normal((n, Hkv, d)), "f16")
        vb = synth.to_bits(rng.standard_normal((n, Hkv, d)), "f16")
        base = int(kv_off[b]) * 2 * Hkv * d
        blk = kv[base: base + n * 2 * Hkv * d].reshape(Hkv, 2, n, d)
        blk[:, 0] = kb.transpose(1, 0, 2)
        blk[:, 1] = vb.transpose(1, 0, 2)
        q = synth.widen(qkv[b:b + 1, :Hq * d], "f16").reshape(1, Hq, d)
        want.append(ofw.causal_attention(q, synth.widen(kb, "f16"), synth.widen(vb, "f16"), lens_before[b]).reshape(1, Hq * d))
    dv = dict(qkv=_dev16(qkv), kv=_dev16(kv), kv_off=_i32(kv_off), cap=_i32(caps), len_before=_i32(lens_before))
    return dv, np.concatenate(want, axis=0), B


def _both(dv, B, Hq, Hkv, d, S, max_len):
    out_a = torch.zeros(B, Hq * d, dtype=torch.int16, device="cuda")
    out_b = torch.full((B, Hq * d), 0x7e00, dtype=torch.int16, device="cuda")
    part = torch.zeros(B * Hq * 16 * (d + 2), dtype=torch.float32, device="cuda")
    K.sn_k_attn_decode(sn.SN_F16, dv["qkv"], dv["kv"], dv["len_before"], dv["kv_off"], dv["cap"], out_a, part, B, Hq, Hkv, d, S, max_len)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    K.sn_k_attn_decode_static(sn.SN_F16, dv["qkv"], dv["kv"], dv["len_before"], dv["kv_off"], dv["cap"], out_b, B, Hq, Hkv, d, S, max_len)
    torch.cuda.synchronize()
    free_after = torch.cuda.mem_get_info()[0]
    return out_a, out_b, free_before, free_after


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 8, 64), (16, 2, 128)])
def test_static_scratch_attention_equals_the_allocating_entry_point(Hq, Hkv, d):
    big = [700, 37, 513, 0, 1290]
    small = [300, 5]
    first = True
    for S in (0, 4, 16, 1):
        for seed, lens in ((1, big), (2, small)):             # the second call is smaller: stale partials lie beyond it
            dv, want, B = _case(seed, lens, Hq, Hkv, d)
            out_a, out_b, f0, f1 = _both(dv, B, Hq, Hkv, d, S, max(lens) + 1)
            assert torch.equal(out_a, out_b), (S, lens)
            if not first:                                        # the very first call may load the code object
                assert f0 == f1, "free device memory moved across a call that must not allocate"
            first = False
            got = synth.widen(out_b.cpu().numpy().view(np.uint16), "f16")
            rms = float(np.sqrt((want ** 2).mean()))
            err = float(np.abs(got - want).max())
            print(f"static attn S={S} B={B}: max|d| = {err / rms:.2e} x RMS", flush=True)
            assert np.isfinite(got).all() and err <= 2e-2 * rms


def test_static_scratch_refuses_what_does_not_fit():
    # 16 key ranges x 512 sequences x 64 heads x 130 floats = 272 MB of partials: beyond the 16 MiB buffer
    dummy = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(sn.SnError) as e:
        K.sn_k_attn_decode_static(sn.SN_F16, dummy, dummy, dummy, dummy, dummy, dummy, 512, 64, 8, 128, 16, 4096)
    assert e.value.code == sn.SN_E_INVAL and "static buffer holds" in str(e.value)
