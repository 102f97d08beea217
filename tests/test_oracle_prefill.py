"""Pins of the oracle's prefill attention against things other than itself.

The paper says only that the prefill phase is that of plain LLM inference
(Section 4; Algorithm 1, Prefill), so what is pinned is textbook causal
self-attention over the prompt: the query at prompt position p reads tokens
0..p.  Pins: dense brute force per query, closed forms (first token, equal
keys), causality, chunked = whole, and the decode oracle on the last token."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from dense_ref import dense_attention
from helpers import make_oracle


def _draw(rng, n, heads, d, dtype):
    x = rng.standard_normal((n, heads, d)).astype(np.float32)
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x)
        return bits, wl.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


def _oracle(Hq=4, Hkv=2, d=16, pt=4, dtype="f32", max_req=2, free_order=None):
    return make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=64, max_req=max_req, Nb=2, max_bp=8, max_pp=16,
                       dtype=dtype, free_order=free_order)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P", [1, 4, 5, 15, 17, 32])      # pt = 4: one token, a page, a page + 1, ragged, aligned
def test_matches_dense_bruteforce_per_query(dtype, P):
    rng = np.random.default_rng(500 + P)
    perm = rng.permutation(64).astype(np.int32)          # scattered pages: the prefix table is really used
    o = _oracle(dtype=dtype, free_order=perm)
    k, kd = _draw(rng, P, 2, 16, dtype)
    v, vd = _draw(rng, P, 2, 16, dtype)
    assert o.append(orc.SEQ_PREFIX, [1], [P], k, v) == orc.OK
    q, qd = _draw(rng, P, 4, 16, dtype)
    out, ws = o.prefill_attention(1, q, want_wsum=True)
    for p in range(P):
        ref = dense_attention(qd[p], kd[:p + 1], vd[:p + 1])
        np.testing.assert_allclose(out[p], ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(ws, 1.0, rtol=0, atol=1e-14)


def test_first_token_returns_its_own_value_and_equal_keys_average():
    rng = np.random.default_rng(7)
    o = _oracle()
    P = 11
    k = np.repeat(rng.standard_normal((1, 2, 16)).astype(np.float32), P, axis=0)     # all keys equal
    v = rng.standard_normal((P, 2, 16)).astype(np.float32)
    assert o.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    q = rng.standard_normal((P, 4, 16)).astype(np.float32)
    out = o.prefill_attention(0, q)
    G = 2
    for h in range(4):
        np.testing.assert_allclose(out[0, h], v[0, h // G].astype(np.float64), rtol=0, atol=1e-15)
        for p in range(P):     # equal scores -> uniform weights -> running mean of V
            np.testing.assert_allclose(out[p, h], v[:p + 1, h // G].astype(np.float64).mean(0), rtol=0, atol=1e-13)


def test_causality_later_tokens_do_not_matter():
    rng = np.random.default_rng(8)
    P, cut = 19, 9
    k, _ = _draw(rng, P, 2, 16, "f32")
    v, _ = _draw(rng, P, 2, 16, "f32")
    q, _ = _draw(rng, P, 4, 16, "f32")
    a = _oracle()
    assert a.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    full = a.prefill_attention(0, q)
    k2, v2 = k.copy(), v.copy()
    k2[cut:] = rng.standard_normal(k2[cut:].shape)       # different future
    v2[cut:] = rng.standard_normal(v2[cut:].shape)
    b = _oracle()
    assert b.append(orc.SEQ_PREFIX, [0], [P], k2, v2) == orc.OK
    other = b.prefill_attention(0, q)
    np.testing.assert_array_equal(full[:cut], other[:cut])
    assert np.abs(full[cut:] - other[cut:]).max() > 1e-3


def test_chunked_prefill_equals_whole_and_last_token_equals_decode():
    rng = np.random.default_rng(9)
    P = 23
    k, _ = _draw(rng, P, 2, 16, "f32")
    v, _ = _draw(rng, P, 2, 16, "f32")
    q, _ = _draw(rng, P, 4, 16, "f32")
    whole = _oracle()
    assert whole.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    ref = whole.prefill_attention(0, q)
    chunked = _oracle()
    got, at = [], 0
    for n in (5, 1, 9, 8):                               # append a chunk, attend with the chunk's queries
        assert chunked.append(orc.SEQ_PREFIX, [0], [n], k[at:at + n], v[at:at + n]) == orc.OK
        got.append(chunked.prefill_attention(0, q[at:at + n]))
        at += n
    np.testing.assert_allclose(np.concatenate(got), ref, rtol=0, atol=1e-14)
    # the last prompt token's query sees the whole prompt: the decode oracle on a branch without private tokens
    dec = whole.attention(np.repeat(q[-1:], 2, axis=0))
    np.testing.assert_allclose(dec[0], ref[-1], rtol=0, atol=1e-14)
    # an empty query chunk is legal and returns nothing
    assert whole.prefill_attention(0, q[:0]).shape == (0, 4, 16)


def test_error_codes():
    rng = np.random.default_rng(10)
    o = _oracle()
    k, _ = _draw(rng, 6, 2, 16, "f32")
    q, _ = _draw(rng, 7, 4, 16, "f32")
    assert o.prefill_attention(1, q[:1]) == orc.E_STATE          # request never created
    assert o.append(orc.SEQ_PREFIX, [1], [6], k, k) == orc.OK
    assert o.prefill_attention(1, q) == orc.E_INVALID            # more queries than prompt tokens
    assert o.prefill_attention(5, q[:1]) == orc.E_INVALID        # no such request slot
    assert o.finish([2, 3]) == orc.OK                            # both branches gone: the prompt is released
    assert o.prefill_attention(1, q[:1]) == orc.E_STATE
