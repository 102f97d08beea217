"""GPU parity of prefill attention (Algorithm 1, Prefill) against the float64
oracle: whole and chunked prefill, every kernel path, edge cases, error codes,
and full-size prompts of the 32B-like and heavy-tail configurations."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import GpuEngine, TOL, dims
from helpers import make_oracle

pytestmark = pytest.mark.gpu


def _pair(cfg, num_pages, max_pp, free_order=None, force_natural_layout=False, max_req=None):
    R = max_req or cfg.n_requests
    o = make_oracle(Hq=cfg.n_q_heads, Hkv=cfg.n_kv_heads, d=cfg.head_dim, pt=cfg.page_tokens, num_pages=num_pages,
                    max_req=R, Nb=cfg.nb, Q=cfg.quota, max_bp=4, max_pp=max_pp, dtype=cfg.dtype, free_order=free_order)
    kw = dims(cfg, num_pages, 4, max_pp=max_pp, max_req=R)
    g = GpuEngine(free_order=free_order, force_natural_layout=force_natural_layout, **kw)
    return o, g


def _check(cfg, o, g, reqs, nqs, qs):
    """One library call for all listed requests against one oracle call each."""
    out = g.c.prefill_attention(reqs, nqs, np.concatenate(qs)).cpu().numpy().astype(np.float64)
    assert g.c.sync_status() == 0
    assert np.all(np.isfinite(out))
    at, worst = 0, 0.0
    for r, n, q in zip(reqs, nqs, qs):
        ref = o.prefill_attention(r, q)
        if n:
            worst = max(worst, float(np.abs(out[at:at + n] - ref).max()))
        at += n
    assert worst <= TOL[cfg.dtype], f"max abs err {worst}"
    return worst


@pytest.mark.parametrize("mode", ["mfma16", "natural"])
@pytest.mark.parametrize("shape", [(28, 4, 128), (40, 8, 128), (8, 2, 64), (16, 1, 128), (64, 8, 128)],
                         ids=["g7", "g5", "g4d64", "g16", "g8-70b"])
def test_whole_and_chunked_prefill_small(shape, mode):
    Hq, Hkv, d = shape
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_requests=5, nb=2, prompt_len=300)
    P = [1, 16, 17, 100, 300]                      # one token, one page, a page + 1, ragged, several row tiles
    pages = sum(-(-p // 16) for p in P) + 4
    o, g = _pair(cfg, pages, 19, free_order=wl.free_order(cfg, pages), force_natural_layout=mode == "natural")
    qs = []
    for r, p in enumerate(P):
        k, v = wl.prefix_kv(cfg, r, p)
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, [r], [p], k, v) == orc.OK
        qs.append(wl.prefix_query(cfg, r, p))
    err = _check(cfg, o, g, list(range(5)), P, qs)
    print(f"{shape} {mode}: whole prefill max abs err {err:.3g}")
    # the last n tokens only (what a chunked prefill asks for), an empty list entry, a request listed alone
    _check(cfg, o, g, [4, 2, 3], [37, 0, 100], [qs[4][-37:], qs[2][:0], qs[3]])
    _check(cfg, o, g, [1], [1], [qs[1][-1:]])
    # a long last chunk after a first chunk (for the wider head groups this takes the 256-row tiles, two per
    # workgroup, with queries that do not start at the prompt's first token), beside a short one
    _check(cfg, o, g, [3, 4], [60, 200], [qs[3][-60:], qs[4][-200:]])


def test_chunked_prefill_append_then_attend():
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=2, nb=2, prompt_len=200)
    o, g = _pair(cfg, 32, 13)
    k = [wl.prefix_kv(cfg, r) for r in range(2)]
    q = [wl.prefix_query(cfg, r) for r in range(2)]
    at = 0
    for n in (16, 1, 70, 113):                    # both requests grow chunk by chunk
        for r in range(2):
            for e in (o, g):
                assert e.append(orc.SEQ_PREFIX, [r], [n], k[r][0][at:at + n], k[r][1][at:at + n]) == orc.OK
        _check(cfg, o, g, [0, 1], [n, n], [q[0][at:at + n], q[1][at:at + n]])
        at += n
    # fp32 cache (natural layout): the benchmark spec's fp32 tolerance
    cfg1 = wl.scaled(wl.CONFIGS[1], n_requests=1, prompt_len=128)
    o, g = _pair(cfg1, 12, 8)
    kk, vv = wl.prefix_kv(cfg1, 0)
    for e in (o, g):
        assert e.append(orc.SEQ_PREFIX, [0], [128], kk, vv) == orc.OK
    err = _check(cfg1, o, g, [0], [128], [wl.prefix_query(cfg1, 0)])
    print(f"fp32 prefill max abs err {err:.3g}")


def test_prefill_errors_are_sticky_and_write_nothing():
    import torch
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=3, nb=2, prompt_len=40)
    o, g = _pair(cfg, 16, 3)
    k, v = wl.prefix_kv(cfg, 1)
    for e in (o, g):
        assert e.append(orc.SEQ_PREFIX, [1], [40], k, v) == orc.OK
    q = wl.prefix_query(cfg, 1, 41)
    out = torch.full((41, cfg.n_q_heads, cfg.head_dim), 7.0, device="cuda")
    # more queries than prompt tokens: found on the device
    g.c.prefill_attention([1], [41], q, out=out)
    assert g.c.sync_status() == orc.E_INVALID and o.prefill_attention(1, q) == orc.E_INVALID
    assert torch.all(out == 7.0)
    # a request that was never created
    g.c.prefill_attention([1, 2], [1, 1], q[:2], out=out[:2])
    assert g.c.sync_status() == orc.E_STATE and o.prefill_attention(2, q[:1]) == orc.E_STATE
    assert torch.all(out == 7.0)
    # host-checkable faults return at once
    assert g.c.prefill_attention([3], [1], q[:1], out=out[:1], status=True) == orc.E_INVALID
    assert g.c.prefill_attention([1], [-1], q[:0], out=out[:0], status=True) == orc.E_INVALID
    # the prompt is released with the request's last branch
    for e in (o, g):
        assert e.finish([2, 3]) == orc.OK
    g.c.prefill_attention([1], [1], q[:1], out=out[:1])
    assert g.c.sync_status() == orc.E_STATE and o.prefill_attention(1, q[:1]) == orc.E_STATE
    assert torch.all(out == 7.0)


@pytest.mark.parametrize("cfg_id,n_req", [(4, 3), (5, 1)])
def test_full_size_prompts(cfg_id, n_req):
    """Prompts of the 32B-like (1024 tokens, G = 5) and heavy-tail (2048 tokens, G = 7) configurations in
    the launch shape bench.py times (whole prompts of several requests in one call)."""
    cfg = wl.scaled(wl.CONFIGS[cfg_id], n_requests=n_req)
    pp = cfg.prompt_len // 16
    pages = n_req * pp + 8
    o, g = _pair(cfg, pages, pp, free_order=wl.free_order(cfg, pages))
    qs = []
    for r in range(n_req):
        k, v = wl.prefix_kv(cfg, r)
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, [r], [cfg.prompt_len], k, v) == orc.OK
        qs.append(wl.prefix_query(cfg, r))
    err = _check(cfg, o, g, list(range(n_req)), [cfg.prompt_len] * n_req, qs)
    print(f"config {cfg_id} prompts: max abs err {err:.3g}")


@pytest.mark.parametrize("slope", [0.25, 0.01])
def test_scores_that_keep_rising(slope):
    """Keys that grow with the position make every page pair raise the row maxima (steeply: by far more than
    the kernel's lag on every pair; gently: by less, so that the reference stays behind for long stretches)."""
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=1, nb=2, prompt_len=300)
    P = cfg.prompt_len
    o, g = _pair(cfg, 24, 19)
    rng = np.random.default_rng(11)
    ramp = (np.arange(P, dtype=np.float32) * slope)[:, None, None]
    k = wl.f32_to_bf16_bits(np.broadcast_to(ramp, (P, cfg.n_kv_heads, cfg.head_dim)).copy())
    v = wl.f32_to_bf16_bits(rng.standard_normal((P, cfg.n_kv_heads, cfg.head_dim)).astype(np.float32))
    for e in (o, g):
        assert e.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    q = wl.f32_to_bf16_bits(np.ones((P, cfg.n_q_heads, cfg.head_dim), np.float32))
    err = _check(cfg, o, g, [0], [P], [q])
    print(f"rising scores, slope {slope}: max abs err {err:.3g}")


@pytest.mark.parametrize("seed", range(8))
def test_random_geometries_and_lengths(seed):
    """Seeded draws of the head geometry, the prompt lengths of five requests (so that the tiles per kv head come
    out odd and even, one and many, with ragged last tiles) and the number of trailing queries of each, attended
    in one call; then the same prompts grown by a random chunk and attended for that chunk only."""
    rng = np.random.default_rng(4242 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.integers(1, 9))
    d = 64 if seed % 4 == 3 else 128
    top = int(rng.choice([90, 260, 700]))
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=d, n_requests=5, nb=2, prompt_len=top + 130)
    P = [int(x) for x in rng.integers(1, top + 1, size=5)]
    grow = [int(x) for x in rng.integers(1, 130, size=5)]
    max_pp = -(-(top + 130) // 16)
    pages = sum(-(-(p + g_) // 16) for p, g_ in zip(P, grow)) + 4
    o, g = _pair(cfg, pages, max_pp, free_order=wl.free_order(cfg, pages))
    kv = [wl.prefix_kv(cfg, r, P[r] + grow[r]) for r in range(5)]
    qs = [wl.prefix_query(cfg, r, P[r] + grow[r]) for r in range(5)]
    for r in range(5):
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, [r], [P[r]], kv[r][0][:P[r]], kv[r][1][:P[r]]) == orc.OK
    nq = [int(rng.integers(0, p + 1)) for p in P]
    nq[int(np.argmax(P))] = max(P)                 # the longest prompt whole: decides the tile size of the call
    order = [int(x) for x in rng.permutation(5)]
    _check(cfg, o, g, order, [nq[r] for r in order], [qs[r][P[r] - nq[r]:P[r]] for r in order])
    for r in range(5):
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, [r], [grow[r]], kv[r][0][P[r]:], kv[r][1][P[r]:]) == orc.OK
    err = _check(cfg, o, g, list(range(5)), grow, [qs[r][P[r]:] for r in range(5)])
    print(f"seed {seed}: Hkv {Hkv} G {G} d {d} prompts {P} + {grow}: max abs err {err:.3g}")
