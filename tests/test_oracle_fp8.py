"""Pins of the oracle's 8-bit float (OCP FP8 E4M3) cache against things other
than itself: the format's definition written out as a table, torch's
float8_e4m3fn conversion (a library's), and the attention of a bf16 cache that
was handed the already rounded values."""
import numpy as np
import pytest
import torch

import oracle as orc
import workloads as wl
from helpers import make_oracle


def _all_bf16_finite():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = wl.bf16_bits_to_f32(bits)
    keep = np.isfinite(vals)
    return bits[keep], vals[keep].astype(np.float64)


def test_codes_decode_as_the_format_defines():
    # feed every exactly representable magnitude: it must come back unchanged with its own code
    for code in range(127):
        e, m = code >> 3, code & 7
        val = (m / 8) * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
        bits = wl.f32_to_bf16_bits(np.array([val, -val], np.float32))
        assert wl.bf16_bits_to_f32(bits)[0] == np.float32(val)          # E4M3 values are exact in bf16
        codes, back = orc.fp8_roundtrip(bits)
        assert codes[0] == code and back[0] == val and back[1] == -val
        if code:
            assert codes[1] == (0x80 | code)
    assert orc.fp8_roundtrip(wl.f32_to_bf16_bits(np.array([448.0], np.float32)))[0][0] == 0x7E   # largest finite


def test_rounding_matches_torch_float8_e4m3fn_on_every_bf16_value():
    bits, vals = _all_bf16_finite()
    codes, back = orc.fp8_roundtrip(bits)
    clamped = np.clip(vals, -448.0, 448.0)               # the cache clamps before it rounds
    ref = torch.from_numpy(clamped.astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(back, ref)
    # nearest: no other code is closer
    table = np.array([orc.fp8_roundtrip(wl.f32_to_bf16_bits(np.array([0.0], np.float32)))[1][0]] +
                     [((c & 7) / 8) * 2.0 ** -6 if (c >> 3) == 0 else (1 + (c & 7) / 8) * 2.0 ** ((c >> 3) - 7) for c in range(1, 127)])
    best = np.abs(np.abs(clamped)[:, None] - table[None, :]).min(1)
    np.testing.assert_array_equal(np.abs(back - clamped), best)
    # a scale divides before rounding and multiplies after
    _, scaled = orc.fp8_roundtrip(bits[::97], scale=0.37)
    with np.errstate(over="ignore"):                     # the largest bf16 values overflow to inf, then clamp to 448
        pre = vals[::97].astype(np.float32) * (np.float32(1.0) / np.float32(0.37))     # float32, like the cache's kernels
    ref2 = torch.from_numpy(np.clip(pre, -448, 448)).to(torch.float8_e4m3fn).to(torch.float32).numpy()
    np.testing.assert_array_equal(scaled, ref2.astype(np.float64) * 0.37)


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.5, 0.25)])
def test_fp8_cache_attends_like_a_bf16_cache_given_the_rounded_values(scales):
    """With power-of-two scales value(code) * scale is itself a bf16 number, so a bf16 oracle cache fed
    those numbers must give the same attention (decode and prefill)."""
    ks, vs = scales
    rng = np.random.default_rng(77)
    kw = dict(Hq=4, Hkv=2, d=16, pt=4, num_pages=64, max_req=1, Nb=2, max_bp=8, max_pp=8)
    a = make_oracle(dtype="fp8", **kw) if ks == 1.0 else orc.OracleCache(
        n_q_heads=4, n_kv_heads=2, head_dim=16, page_tokens=4, num_pages=64, max_requests=1, branches_per_request=2,
        finish_quota=0, max_pages_per_branch=8, max_prefix_pages=8, dtype="fp8", k_scale=ks, v_scale=vs)
    b = make_oracle(dtype="bf16", **kw)

    def draw(n):
        x = wl.f32_to_bf16_bits((rng.standard_normal((n, 2, 16)) * 3).astype(np.float32))
        return x

    def rounded(x, s):
        return wl.f32_to_bf16_bits(orc.fp8_roundtrip(x, s)[1].astype(np.float32))

    for kind, ids, n in ((orc.SEQ_PREFIX, [0], 9), (orc.SEQ_BRANCH, [0], 5), (orc.SEQ_BRANCH, [1], 14)):
        k, v = draw(n), draw(n)
        assert a.append(kind, ids, [n], k, v) == orc.OK
        assert b.append(kind, ids, [n], rounded(k, ks), rounded(v, vs)) == orc.OK
    q = wl.f32_to_bf16_bits(rng.standard_normal((2, 4, 16)).astype(np.float32))
    np.testing.assert_allclose(a.attention(q), b.attention(q), rtol=0, atol=1e-13)
    qp = wl.f32_to_bf16_bits(rng.standard_normal((9, 4, 16)).astype(np.float32))
    np.testing.assert_allclose(a.prefill_attention(0, qp), b.prefill_attention(0, qp), rtol=0, atol=1e-13)
