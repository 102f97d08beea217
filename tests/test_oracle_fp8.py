"""Pins of the oracle's 8-bit float (OCP FP8 E4M3) cache against things other
than itself: the format's definition written out as a table, torch's
float8_e4m3fn conversion (a library's), exact rational arithmetic for scaled
values (with hand-worked ties), and the attention of a bf16 cache that was
handed the already rounded values."""
from fractions import Fraction

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


def _e4m3_table():
    """The 127 finite magnitudes by code, as exact fractions (the format's definition)."""
    return [Fraction(c & 7, 8) * Fraction(1, 64) if (c >> 3) == 0 else (1 + Fraction(c & 7, 8)) * Fraction(2) ** ((c >> 3) - 7)
            for c in range(127)]


def _exact_code(x, scale, table):
    """Nearest code of |x / scale| in exact rational arithmetic, ties to the even code, clamped to 448."""
    t = min(abs(Fraction(float(x)) / Fraction(float(scale))), Fraction(448))
    return min(range(127), key=lambda c: (abs(table[c] - t), c & 1))


def test_scaled_codes_are_those_of_the_exact_quotient():
    """code = nearest(x / scale): checked against exact rational arithmetic (no floating point decides
    anything), on every bf16 value of eight binades for scales where float32 short-cuts go wrong."""
    table = _e4m3_table()
    # hand-worked ties.  91/1024 / 7 = 13/1024 = 6.5 * 2^-9: halfway between subnormal codes 6 and 7, so the even
    # code 6; 175/1024 / 7 = 25/1024 = 12.5 * 2^-9: halfway between codes 12 and 13 ((8 + m) * 2^-9 in that
    # binade), so 12.  Multiplying by the float32 reciprocal of 7 (which is above 1/7) lands above both ties.
    for num, want in ((91, 6), (175, 12)):
        x = np.float32(num / 1024.0)
        bits = wl.f32_to_bf16_bits(np.array([x, -x], np.float32))
        assert wl.bf16_bits_to_f32(bits)[0] == x                       # exact in bf16
        codes, back = orc.fp8_roundtrip(bits, scale=7.0)
        assert list(codes) == [want, 0x80 | want]
        assert back[0] == float(table[want]) * 7.0
        recip = np.float32(x) * (np.float32(1.0) / np.float32(7.0))    # the short-cut, for contrast
        assert _exact_code(recip, 1.0, table) == want + 1
    # every bf16 value from 2^-7 up to 2^1, four scales (float32 values, as a cache description carries them)
    bits = np.arange(0x3C00, 0x4000, dtype=np.uint32).astype(np.uint16)
    bits = np.concatenate([bits, bits | 0x8000])
    vals = wl.bf16_bits_to_f32(bits)
    n_recip = n_div32 = 0
    for scale in (7.0, 0.37, 1.7, 0.011):
        s32 = np.float32(scale)
        codes, back = orc.fp8_roundtrip(bits, scale=scale)
        want = np.array([_exact_code(x, s32, table) for x in vals])
        np.testing.assert_array_equal(codes & 0x7F, want)
        np.testing.assert_array_equal((codes & 0x80) != 0, np.signbit(vals))
        np.testing.assert_array_equal(back, np.where(np.signbit(vals), -1.0, 1.0) *
                                      np.array([float(table[c]) for c in want]) * float(s32))
        # the pin tells the definitions apart: both float32 short-cuts decide some of these codes differently
        n_recip += sum(_exact_code(x * (np.float32(1.0) / s32), 1.0, table) != w for x, w in zip(vals, want))
        n_div32 += sum(_exact_code(x / s32, 1.0, table) != w for x, w in zip(vals, want))
    assert n_recip > 0 and n_div32 > 0, (n_recip, n_div32)


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
