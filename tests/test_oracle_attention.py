"""Pins of the oracle's attention and paging against things other than itself:
dense brute force, closed forms, invariances and a library softmax.

The paper gives no attention formula of its own (Section 4: prefill and decode
are those of vanilla LLM inference; Section 2: one token per decode step), so
the definition being pinned is the textbook softmax(q K^T / sqrt(d)) V."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle as orc
import workloads as wl
from dense_ref import dense_attention
from helpers import DenseShadow, check_invariants, make_oracle


def _build(rng, *, Hq=4, Hkv=2, d=16, pt=4, P=7, Ls=(1, 4, 5, 9), dtype="f32", num_pages=64, free_order=None,
           max_bp=16, max_pp=8):
    """One request with len(Ls) branches; returns (oracle, shadow, q raw)."""
    Nb = len(Ls)
    o = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=num_pages, max_req=1, Nb=Nb, max_bp=max_bp,
                    max_pp=max_pp, dtype=dtype, free_order=free_order)
    sh = DenseShadow(Hkv, d)

    def draw(n):
        x = rng.standard_normal((n, Hkv, d)).astype(np.float32)
        if dtype == "bf16":
            bits = wl.f32_to_bf16_bits(x)
            return bits, wl.bf16_bits_to_f32(bits).astype(np.float64)
        return x, x.astype(np.float64)

    k, kd = draw(P)
    v, vd = draw(P)
    assert o.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    sh.add_prefix(0, kd, vd)
    for j, L in enumerate(Ls):
        k, kd = draw(L)
        v, vd = draw(L)
        assert o.append(orc.SEQ_BRANCH, [j], [L], k, v) == orc.OK
        sh.add_private(j, kd, vd)
    qf = rng.standard_normal((Nb, Hq, d)).astype(np.float32)
    if dtype == "bf16":
        q = wl.f32_to_bf16_bits(qf)
        qd = wl.bf16_bits_to_f32(q).astype(np.float64)
    else:
        q, qd = qf, qf.astype(np.float64)
    return o, sh, q, qd


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P,Ls", [
    (0, (1, 4, 5, 9)),      # no prompt; L = 1, pt, pt+1
    (1, (3, 8, 1, 2)),
    (15, (16, 17, 1, 4)),   # prompt one short of 4 pages (pt=4): 15 = 3*4+3
    (17, (4, 4, 4, 33)),
    (8, (12, 1, 7, 20)),    # page-aligned prompt
])
def test_P1_matches_dense_bruteforce(dtype, P, Ls):
    rng = np.random.default_rng(100 + P)
    o, sh, q, qd = _build(rng, P=P, Ls=Ls, dtype=dtype)
    out, ws = o.attention(q, want_wsum=True)
    for a in range(len(Ls)):
        K, V = sh.context(a, len(Ls))
        assert K.shape[0] == P + Ls[a]
        ref = dense_attention(qd[a], K, V)
        np.testing.assert_allclose(out[a], ref, rtol=0, atol=1e-12)
    # P2: softmax weights sum to one
    np.testing.assert_allclose(ws, 1.0, rtol=0, atol=1e-14)
    check_invariants(o.state(), pt=4, num_pages=64, Nb=len(Ls), max_req=1)


def test_P1_gqa_head_mapping_and_scale():
    """Query head h must read KV head h // G, and an explicit scale is used as given."""
    rng = np.random.default_rng(7)
    o, sh, q, qd = _build(rng, Hq=6, Hkv=3, d=8, P=5, Ls=(3, 6))
    out = o.attention(q, scale=0.37)
    for a in range(2):
        K, V = sh.context(a, 2)
        np.testing.assert_allclose(out[a], dense_attention(qd[a], K, V, scale=0.37), atol=1e-12)
    # a wrong head map would give a different answer here
    K, V = sh.context(0, 2)
    wrong = dense_attention(qd[0], K[:, ::-1], V[:, ::-1], scale=0.37)
    assert np.abs(wrong - out[0]).max() > 1e-3


def test_P8_library_softmax_single_branch():
    """One branch, no prompt: equals scipy's softmax followed by a matmul."""
    rng = np.random.default_rng(8)
    o, sh, q, qd = _build(rng, Hq=2, Hkv=1, d=32, pt=16, P=0, Ls=(37,), max_bp=4)
    out = o.attention(q)
    K, V = sh.context(0, 1)
    for h in range(2):
        w = softmax(K[:, 0, :] @ qd[0, h] / np.sqrt(32.0))
        np.testing.assert_allclose(out[0, h], w @ V[:, 0, :], atol=1e-13)


def test_P3_shared_prefix_equals_duplicated_private_copy():
    """The prompt stored once and shared gives the same output as the prompt
    copied in front of every branch's private tokens."""
    rng = np.random.default_rng(3)
    Hq, Hkv, d, pt, P, Ls = 4, 2, 16, 4, 10, (3, 9, 1)
    o, sh, q, _ = _build(rng, Hq=Hq, Hkv=Hkv, d=d, pt=pt, P=P, Ls=Ls, max_bp=16)
    shared = o.attention(q)
    dup = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=64, max_req=1, Nb=len(Ls), max_bp=16, max_pp=8)
    z = np.zeros((0, Hkv, d), np.float32)
    assert dup.append(orc.SEQ_PREFIX, [0], [0], z, z) == orc.OK
    for j in range(len(Ls)):
        K, V = sh.context(j, len(Ls))
        assert dup.append(orc.SEQ_BRANCH, [j], [K.shape[0]], K.astype(np.float32), V.astype(np.float32)) == orc.OK
    np.testing.assert_allclose(dup.attention(q), shared, rtol=0, atol=1e-13)


def test_P6_closed_forms():
    Hq, Hkv, d, pt = 2, 1, 8, 4
    rng = np.random.default_rng(6)
    T = 11
    z = np.zeros((0, Hkv, d), np.float32)

    def run(K, V, q):
        o = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=16, max_req=1, Nb=1, max_bp=8, max_pp=2)
        assert o.append(orc.SEQ_PREFIX, [0], [0], z, z) == orc.OK
        assert o.append(orc.SEQ_BRANCH, [0], [T], K, V) == orc.OK
        return o.attention(q)[0]

    q = rng.standard_normal((1, Hq, d)).astype(np.float32)
    V = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    # (i) all keys equal -> uniform weights -> mean of V
    K = np.tile(rng.standard_normal((1, Hkv, d)).astype(np.float32), (T, 1, 1))
    out = run(K, V, q)
    np.testing.assert_allclose(out, np.tile(V[:, 0].astype(np.float64).mean(0), (Hq, 1)), atol=1e-13)
    # (ii) all V rows equal c -> c
    K = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    c = rng.standard_normal((1, Hkv, d)).astype(np.float32)
    out = run(K, np.tile(c, (T, 1, 1)), q)
    np.testing.assert_allclose(out, np.tile(c[0].astype(np.float64), (Hq, 1)), atol=1e-13)
    # (iii) one key strongly aligned with q (both heads share q here) -> its V row
    q1 = np.tile(q[:, :1], (1, Hq, 1))
    K = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    K[5, 0] = 200.0 * q1[0, 0]
    out = run(K, V, q1)
    np.testing.assert_allclose(out, np.tile(V[5].astype(np.float64), (Hq, 1)), atol=1e-9)
    # (iv) convex hull: per-coordinate min <= out <= max
    K = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    out = run(K, V, q)
    assert np.all(out <= V[:, 0].max(0) + 1e-12) and np.all(out >= V[:, 0].min(0) - 1e-12)
    # two tokens, hand-computed: scores s0, s1 -> weights 1/(1+e^(s1-s0)), ...
    T = 2
    K2 = np.zeros((2, 1, d), np.float32); K2[0, 0, 0] = 1.0; K2[1, 0, 0] = 3.0
    V2 = np.zeros((2, 1, d), np.float32); V2[0, 0, 0] = 10.0; V2[1, 0, 1] = -4.0
    q2 = np.zeros((1, Hq, d), np.float32); q2[0, :, 0] = 2.0
    out = run(K2, V2, q2)
    s = np.array([2.0, 6.0]) / np.sqrt(d)
    w1 = 1.0 / (1.0 + np.exp(s[0] - s[1]))
    np.testing.assert_allclose(out[0, :2], [10.0 * (1 - w1), -4.0 * w1], atol=1e-13)


def test_P7_invariances_physical_pages_and_token_order():
    rng = np.random.default_rng(77)
    kw = dict(Hq=4, Hkv=2, d=16, pt=4, P=9, Ls=(5, 13, 2), num_pages=32)
    o1, sh, q, _ = _build(np.random.default_rng(1), **kw)
    perm = rng.permutation(32).astype(np.int32)
    o2, _, q2, _ = _build(np.random.default_rng(1), free_order=perm, **kw)
    assert np.array_equal(q, q2)
    s1, s2 = o1.state(), o2.state()
    assert not np.array_equal(s1["block_tables"], s2["block_tables"])  # really different pages
    np.testing.assert_array_equal(o1.attention(q), o2.attention(q))
    # permuting private tokens of a branch (P=0 so the whole context) leaves out unchanged up to rounding
    Hq, Hkv, d, pt, T = 2, 1, 8, 4, 14
    K = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    V = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    qq = rng.standard_normal((1, Hq, d)).astype(np.float32)
    z = np.zeros((0, Hkv, d), np.float32)
    outs = []
    for order in (np.arange(T), rng.permutation(T)):
        o = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=8, max_req=1, Nb=1, max_bp=8, max_pp=1)
        o.append(orc.SEQ_PREFIX, [0], [0], z, z)
        o.append(orc.SEQ_BRANCH, [0], [T], K[order], V[order])
        outs.append(o.attention(qq))
    np.testing.assert_allclose(outs[0], outs[1], atol=1e-13)


def test_P7_split_merge_algebra():
    """Any split of the context into chunks, each reduced to (m, l, o) and
    merged by m = max m_i, l = sum l_i e^(m_i-m), o = sum o_i e^(m_i-m) / l,
    reproduces the unsplit result (the rule the split-K kernels rely on)."""
    rng = np.random.default_rng(5)
    d, T = 16, 50
    K = rng.standard_normal((T, d)); V = rng.standard_normal((T, d)); q = rng.standard_normal(d)
    o, sh_q = None, None
    oc = make_oracle(Hq=1, Hkv=1, d=d, pt=4, num_pages=16, max_req=1, Nb=1, max_bp=16, max_pp=1)
    z = np.zeros((0, 1, d), np.float32)
    oc.append(orc.SEQ_PREFIX, [0], [0], z, z)
    Kf, Vf, qf = K.astype(np.float32), V.astype(np.float32), q.astype(np.float32)
    oc.append(orc.SEQ_BRANCH, [0], [T], Kf[:, None], Vf[:, None])
    full = oc.attention(qf[None, None])[0, 0]
    cuts = [0, 3, 4, 20, 21, 50]
    parts = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        s = (Kf[a:b].astype(np.float64) @ qf.astype(np.float64)) / np.sqrt(d)
        m = s.max(); e = np.exp(s - m)
        parts.append((m, e.sum(), e @ Vf[a:b].astype(np.float64)))
    m = max(p[0] for p in parts)
    l = sum(p[1] * np.exp(p[0] - m) for p in parts)
    acc = sum(p[2] * np.exp(p[0] - m) for p in parts)
    np.testing.assert_allclose(acc / l, full, atol=1e-13)


def test_empty_context_gives_zero_row():
    o = make_oracle(Hq=2, Hkv=1, d=8, pt=4, num_pages=4, max_req=1, Nb=2, max_bp=2, max_pp=1)
    z = np.zeros((0, 1, 8), np.float32)
    assert o.append(orc.SEQ_PREFIX, [0], [0], z, z) == orc.OK
    out, ws = o.attention(np.ones((2, 2, 8), np.float32), want_wsum=True)
    assert np.all(out == 0) and np.all(ws == 0) and np.all(np.isfinite(out))


def test_bf16_bit_conversion_matches_torch():
    """The generator's bf16 rounding is round-to-nearest-even (checked against torch)."""
    import torch
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.3895314e38]  # ties and near-overflow
    bits = wl.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, t)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(bits),
                                  torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())
