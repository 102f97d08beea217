"""GPU parity: the HIP library against the float64 oracle, through the C ABI.

Integer state (block tables, free stack, active list, lengths, states,
counters) must be bit-exact; attention within 1e-5 (fp32) / 1e-2 (bf16)."""
import json
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import TOL, GpuEngine, compare_attention, dims, populate
from helpers import assert_state_equal, check_invariants, run_golden_scenario

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bookkeeping_small.json")
with open(GOLDEN) as f:
    SCENARIOS = json.load(f)["scenarios"]


def _pair(cfg, num_pages, max_bp, free_order=None, max_pp=None, max_req=None, **gpu_kw):
    kw = dims(cfg, num_pages, max_bp, max_pp, max_req)
    o = orc.OracleCache(free_order=free_order, **kw)
    g = GpuEngine(free_order=free_order, **kw, **gpu_kw)
    return o, g


# ---------------------------------------------------------------------------
# bookkeeping
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("scn", SCENARIOS, ids=[s["name"] for s in SCENARIOS])
def test_golden_traces_on_gpu(scn):
    d = scn["desc"]
    g = GpuEngine(n_q_heads=2, n_kv_heads=1, head_dim=8, page_tokens=d["pt"], num_pages=d["num_pages"],
                  max_requests=d["max_req"], branches_per_request=d["Nb"], finish_quota=d["Q"],
                  max_pages_per_branch=d["max_bp"], max_prefix_pages=d["max_pp"], dtype="f32",
                  start_waiting=d.get("start_waiting", False))
    run_golden_scenario(scn, g, 1, 8, np.float32)


@pytest.mark.parametrize("dtype,pt,d", [("f32", 4, 8), ("bf16", 16, 64)])
def test_random_op_sequences_bit_exact(dtype, pt, d):
    """Random append / prune / finish sequences (errors included): status and
    the whole integer state agree with the oracle after every call."""
    rng = np.random.default_rng(2024)
    R, Nb, num_pages, max_bp, max_pp = 5, 4, 120, 6, 3
    npd = np.float32 if dtype == "f32" else np.uint16
    for trial in range(6):
        kw = dict(n_q_heads=2, n_kv_heads=1, head_dim=d, page_tokens=pt, num_pages=num_pages, max_requests=R,
                  branches_per_request=Nb, finish_quota=int(rng.integers(0, 4)), max_pages_per_branch=max_bp,
                  max_prefix_pages=max_pp, dtype=dtype)
        fo = rng.permutation(num_pages).astype(np.int32) if trial % 2 else None
        o, g = orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)
        ones = lambda n: np.ones((n, 1, d), npd)
        next_req = 0
        for step in range(40):
            st = o.state()
            nA = int(st["n_active"][0])
            op = int(rng.integers(0, 6))
            if op == 0 and next_req < R:
                n = int(rng.integers(0, max_pp * pt + 3))       # sometimes over the prompt capacity
                args = ("append", orc.SEQ_PREFIX, [next_req], [n], ones(n), ones(n))
                next_req += 1
            elif op in (1, 2) and nA:
                if rng.random() < 0.5:
                    n = rng.integers(0, 2 * pt, size=nA)
                    args = ("append", orc.SEQ_BRANCH, None, n, ones(int(n.sum())), ones(int(n.sum())))
                else:
                    m = int(rng.integers(1, nA + 1))
                    ids = rng.choice(R * Nb, size=m, replace=False)   # may hit branches that are not active
                    n = rng.integers(0, 2 * pt, size=m)
                    args = ("append", orc.SEQ_BRANCH, ids, n, ones(int(n.sum())), ones(int(n.sum())))
            elif op == 3 and nA:
                sc = rng.random(nA + int(rng.integers(0, 3))).astype(np.float32)
                sc[rng.integers(0, nA, size=2)] = 0.5
                args = ("prune", int(rng.integers(0, 3)), sc, int(rng.integers(0, 3)),
                        rng.random(R).astype(np.float32), rng.integers(0, Nb + 1, size=R))
            elif op == 4 and nA:
                m = int(rng.integers(1, min(nA, 3) + 1))
                pool = st["active_handles"][:nA] if rng.random() < 0.8 else np.arange(R * Nb)
                args = ("finish", rng.choice(pool, size=m, replace=False))
            else:
                continue
            if args[0] == "append":
                rc_o, rc_g = o.append(*args[1:]), g.append(*args[1:])
            elif args[0] == "prune":
                mode, sc, k, th, mp = args[1:]
                use_cap = rng.random() < 0.5 or mode == 2
                kwp = dict(k=k, threshold=th, max_pruned=mp if use_cap else None)
                rc_o, rc_g = o.prune(mode, sc, **kwp), g.prune(mode, sc, **kwp)
            else:
                rc_o, rc_g = o.finish(args[1]), g.finish(args[1])
            assert rc_o == rc_g, (trial, step, args[0], rc_o, rc_g)
            so, sg = o.state(), g.state()
            assert_state_equal(so, sg)
            check_invariants(sg, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)


# ---------------------------------------------------------------------------
# attention
# ---------------------------------------------------------------------------
def test_cfg1_tiny_decode_prune_decode():
    """Config 1: fp32, 1 request x 4 branches, prompt 128, L ~ U[1,256]; one
    decode step, keep the top 2 by score, decode again."""
    cfg = wl.CONFIGS[1]
    L = wl.lengths(cfg)
    o, g = _pair(cfg, wl.pages_needed(cfg, L) + 8, 17)
    populate(cfg, [o, g], L)
    e1 = compare_attention(cfg, o, g, wl.query(cfg, 0))
    sc = wl.scores(cfg, 0)
    assert o.prune(orc.KEEP_TOP_K, sc, k=2) == orc.OK
    assert g.prune(orc.KEEP_TOP_K, sc, k=2) == orc.OK
    assert_state_equal(o.state(), g.state())
    assert o.state()["n_active"][0] == 2
    e2 = compare_attention(cfg, o, g, wl.query(cfg, 1))
    print(f"cfg1 max abs err {e1:.3g} / {e2:.3g}")


@pytest.mark.parametrize("mode", ["mfma16-per-branch", "mfma16-shared-rows", "natural"])
@pytest.mark.parametrize("shape", [(28, 4, 128), (40, 8, 128), (8, 2, 64), (16, 1, 128), (64, 8, 128)],
                         ids=["g7", "g5", "g4d64", "g16", "g8-70b"])
def test_bf16_small_all_rows(shape, mode):
    """7B-like / 32B-like head geometry at a size the oracle finishes in
    seconds: several pages per branch, ragged tails, a prompt that is not a
    page multiple, one branch with a single token."""
    Hq, Hkv, d = shape
    natural = mode == "natural"
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_requests=3, nb=5, prompt_len=100,
                    length_params=(200, 0.8), length_cap=1500)
    L = wl.lengths(cfg)
    L[0, 0], L[0, 1], L[1, 0] = 1, 16, 17
    o, g = _pair(cfg, wl.pages_needed(cfg, L) + 4, int(-(-L.max() // 16)) + 1,
                 free_order=wl.free_order(cfg, wl.pages_needed(cfg, L) + 4), force_natural_layout=natural)
    assert g.c.layout == (0 if natural else 1)
    pmode = {"mfma16-per-branch": 1, "mfma16-shared-rows": 2, "natural": 1}[mode]
    g.c.set_decode_launch(prompt_mode=pmode)
    populate(cfg, [o, g], L)
    assert_state_equal(o.state(), g.state())
    err = compare_attention(cfg, o, g, wl.query(cfg, 0))
    print(f"shape {shape} {mode}: max abs err {err:.3g}")
    # other launch shapes cut the unit line elsewhere; the result must not depend on it
    for n_wg, skew in ((3, 45), (64, 300), (1000, -200), (256, 0), (1, 50)):
        g.c.set_decode_launch(n_wg, pmode, skew)
        for in_kernel in (False, True):        # the merge kernel / the attention kernel's last writers
            g.c.set_merge_mode(in_kernel)
            compare_attention(cfg, o, g, wl.query(cfg, 1))


def test_edge_cases_empty_and_short_contexts():
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=3, nb=2, prompt_len=0)
    o, g = _pair(cfg, 64, 4, max_pp=2)
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim), np.uint16)
    for e in (o, g):
        assert e.append(orc.SEQ_PREFIX, [0], [0], z, z) == orc.OK      # request 0: no prompt
    k, v = wl.prefix_kv(cfg, 1, 5)
    for e in (o, g):
        assert e.append(orc.SEQ_PREFIX, [1], [5], k, v) == orc.OK      # request 1: 5-token prompt
    kb, vb = wl.branch_kv(cfg, 1, 33)
    for e in (o, g):
        assert e.append(orc.SEQ_BRANCH, [1], [33], kb, vb) == orc.OK   # only branch 1 has private tokens
    # rows: b0 empty context; b1 33 private; b2, b3 prompt only
    q = wl.query(cfg, 0)
    compare_attention(cfg, o, g, q)
    out = g.c.decode_attention(q[:4]).cpu().numpy()
    assert np.all(out[0] == 0)
    # a row buffer smaller than the active list is refused and nothing is written
    import torch
    small = torch.full((3, cfg.n_q_heads, cfg.head_dim), 7.0, device="cuda")
    qd = g.c._dev(q[:3], (cfg.n_q_heads, cfg.head_dim))
    g.c.decode_attention(qd, out=small)
    assert g.c.sync_status() == orc.E_INVALID
    assert torch.all(small == 7.0)
    # the error is cleared once read; the next call works
    compare_attention(cfg, o, g, q)


def test_prune_keeps_survivor_outputs_and_prefix_sharing_on_gpu():
    """Spec invariants on the GPU: survivors' outputs unchanged by
    pruning + compaction; shared prompt equals a per-branch private copy."""
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=2, nb=8, prompt_len=64, length_params=(120, 0.8), length_cap=600)
    L = wl.lengths(cfg)
    o, g = _pair(cfg, wl.pages_needed(cfg, L) + 4, 40)
    populate(cfg, [o, g], L)
    q = wl.query(cfg, 0)
    before = g.c.decode_attention(q).cpu().numpy()
    sc = wl.scores(cfg, 0)
    assert g.prune(orc.DROP_LOWEST_K, sc, k=3) == orc.OK and o.prune(orc.DROP_LOWEST_K, sc, k=3) == orc.OK
    st = g.state()
    assert_state_equal(o.state(), st)
    surv = st["active_handles"][:int(st["n_active"][0])]
    after = g.c.decode_attention(q[surv]).cpu().numpy()
    # same data, same order; only the split points move, and with them the running max that the
    # bf16-rounded softmax weights are taken against
    np.testing.assert_allclose(after, before[surv], rtol=0, atol=2e-3)
    compare_attention(cfg, o, g, q)
    # duplicated-prefix cache
    cfg0 = wl.scaled(cfg, prompt_len=0)
    g2 = GpuEngine(**dims(cfg0, wl.pages_needed(cfg, L) + 16 * 8 + 4, 48, max_pp=1))
    z = np.zeros((0, cfg.n_kv_heads, cfg.head_dim), np.uint16)
    for r in range(cfg.n_requests):
        assert g2.append(orc.SEQ_PREFIX, [r], [0], z, z) == orc.OK
        pk, pv = wl.prefix_kv(cfg, r)
        for j in range(cfg.nb):
            b = r * cfg.nb + j
            kb, vb = wl.branch_kv(cfg, b, int(L[r, j]))
            assert g2.append(orc.SEQ_BRANCH, [b], [64 + int(L[r, j])], np.concatenate([pk, kb]),
                             np.concatenate([pv, vb])) == orc.OK
    dup = g2.c.decode_attention(q).cpu().numpy()
    np.testing.assert_allclose(dup, before, rtol=0, atol=2e-3)


# ---------------------------------------------------------------------------
# full-size configurations (the launch shape bench.py times), sampled rows
# ---------------------------------------------------------------------------
def _request_arrays(cfg, r, L):
    pk, pv = wl.prefix_kv(cfg, r)
    ids = [r * cfg.nb + j for j in range(cfg.nb)]
    ns = [int(L[r, j]) for j in range(cfg.nb)]
    kv = [wl.branch_kv(cfg, b, n) for b, n in zip(ids, ns)]
    return r, pk, pv, ids, ns, np.concatenate([x[0] for x in kv]), np.concatenate([x[1] for x in kv])


class _IntegerShadow:
    """The oracle's bookkeeping at full size without the KV bytes: integer state (free stack, tables, lengths,
    states, counters) does not depend on the head geometry, so a second oracle cache with ONE kv head of
    8 elements, the same pool size, free order, limits and call sequence, fed zeros, holds exactly the state
    the real-size cache must hold."""

    def __init__(self, cfg, num_pages, max_bp, free_order):
        tiny = wl.scaled(cfg, n_q_heads=1, n_kv_heads=1, head_dim=8)
        self.o = orc.OracleCache(free_order=free_order, **dims(tiny, num_pages, max_bp))

    def append(self, kind, ids, ns, k, v):
        n = int(np.sum(ns)) if ns is not None else (len(ids) if ids is not None else self.o.n_active)
        z = np.zeros((n, 1, 8), np.uint16)
        return self.o.append(kind, ids, ns, z, z)

    def prune(self, *a, **kw):
        return self.o.prune(*a, **kw)

    def state(self):
        return self.o.state()


def _populate_full(cfg, g, o, shadow, L, sample_reqs):
    """All requests go to the GPU cache and to the integer shadow; only the sampled ones to the attention
    oracle (attention does not depend on which physical pages hold the tokens)."""
    with ThreadPoolExecutor(max_workers=8) as ex:
        for r, pk, pv, ids, ns, bk, bv in ex.map(lambda r: _request_arrays(cfg, r, L), range(cfg.n_requests)):
            for e in ([g, o, shadow] if r in sample_reqs else [g, shadow]):
                assert e.append(orc.SEQ_PREFIX, [r], [cfg.prompt_len], pk, pv) == orc.OK
                assert e.append(orc.SEQ_BRANCH, ids, ns, bk, bv) == orc.OK


@pytest.mark.parametrize("cfg_id,sample", [(2, (0, 7, 15)), (4, (3, 40)), (5, (0,))])
def test_full_size_configs_sampled_rows(cfg_id, sample):
    """Configurations 2, 4 and 5 at full size in the launch shape bench.py times: the whole integer state
    bit-exact against the oracle's bookkeeping (after the build, after a decode step's append, and for
    configuration 5 after keeping the top 16 of 64 branches), attention on sampled requests."""
    cfg = wl.CONFIGS[cfg_id]
    L = wl.lengths(cfg)
    num_pages = wl.pages_needed(cfg, L, growth_tokens=1) + 64
    max_bp = cfg.length_cap // 16 + 1
    fo = wl.free_order(cfg, num_pages)
    g = GpuEngine(free_order=fo, **dims(cfg, num_pages, max_bp))
    shadow = _IntegerShadow(cfg, num_pages, max_bp, fo)
    Ls = L[list(sample)]
    o = orc.OracleCache(**dims(cfg, int(np.sum((Ls + 16) // 16)) + len(sample) * (cfg.prompt_len // 16) + 8, max_bp))
    _populate_full(cfg, g, o, shadow, L, set(sample))
    stg = g.state()
    check_invariants(stg, pt=16, num_pages=num_pages, Nb=cfg.nb, max_req=cfg.n_requests)
    assert_state_equal(shadow.state(), stg)
    q = wl.query(cfg, 0)

    def compare(tag):
        stg, sto = g.state(), o.state()
        assert_state_equal(shadow.state(), stg)                  # all 11 arrays, bit for bit
        nA, nO = int(stg["n_active"][0]), int(sto["n_active"][0])
        act_g = list(stg["active_handles"][:nA])
        act_o = sto["active_handles"][:nO]
        np.testing.assert_array_equal(stg["seq_lens"][[act_g.index(b) for b in act_o]], sto["seq_lens"][:nO])
        out = g.c.decode_attention(q[act_g]).cpu().numpy().astype(np.float64)
        assert g.c.sync_status() == 0 and np.all(np.isfinite(out))
        ref = o.attention(q[act_o])
        err = np.abs(out[[act_g.index(b) for b in act_o]] - ref).max()
        print(f"cfg{cfg_id} {tag}: {nA} rows, {nO} sampled, max abs err {err:.3g}")
        assert err <= TOL[cfg.dtype]

    compare("built")
    # a decode step: one token for every active branch (some cross into a new page), then attention
    k, v = wl.step_kv(cfg, 1)
    act = stg["active_handles"][:int(stg["n_active"][0])]
    act_o = o.state()["active_handles"][:int(o.state()["n_active"][0])]
    assert g.append(orc.SEQ_BRANCH, None, None, k[act], v[act]) == orc.OK
    assert shadow.append(orc.SEQ_BRANCH, None, None, None, None) == orc.OK
    assert o.append(orc.SEQ_BRANCH, None, None, k[act_o], v[act_o]) == orc.OK
    compare("after a step's append")
    if cfg_id == 5:  # prune to 16 branches by score, then decode again
        sc = wl.scores(cfg, 0)
        for e in (g, o, shadow):
            assert e.prune(orc.KEEP_TOP_K, sc, k=16) == orc.OK
        assert int(g.state()["n_active"][0]) == 16
        check_invariants(g.state(), pt=16, num_pages=num_pages, Nb=cfg.nb, max_req=cfg.n_requests)
        compare("after keeping the top 16")


# ---------------------------------------------------------------------------
# many branches: the planning kernels loop over the active list in chunks of
# 1024 rows and search the unit line from LDS only up to 4096 rows
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("R,Nb,dtype", [(300, 8, "bf16"), (1300, 4, "bf16"), (700, 3, "f32")])
def test_many_branches_state_and_attention(R, Nb, dtype):
    rng = np.random.default_rng(R)
    d, Hq, Hkv, pt = 64, 4, 2, 16
    num_pages = R * Nb * 3 + R * 2 + 64
    kw = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, page_tokens=pt, num_pages=num_pages, max_requests=R,
              branches_per_request=Nb, finish_quota=2, max_pages_per_branch=4, max_prefix_pages=2, dtype=dtype)
    fo = rng.permutation(num_pages).astype(np.int32)
    o, g = orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)

    def draw(n, heads):
        x = rng.standard_normal((n, heads, d)).astype(np.float32)
        return x if dtype == "f32" else wl.f32_to_bf16_bits(x)

    P = rng.integers(0, 2 * pt + 1, size=R)
    for r0 in range(0, R, 64):                      # prompts, 64 requests per call
        ids = np.arange(r0, min(R, r0 + 64))
        k, v = draw(int(P[ids].sum()), Hkv), draw(int(P[ids].sum()), Hkv)
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, ids, P[ids], k, v) == orc.OK
    L = rng.integers(0, 3 * pt, size=R * Nb)        # some branches stay empty
    k, v = draw(int(L.sum()), Hkv), draw(int(L.sum()), Hkv)
    for e in (o, g):
        assert e.append(orc.SEQ_BRANCH, None, L, k, v) == orc.OK
    assert_state_equal(o.state(), g.state())
    q = draw(R * Nb, Hq)
    rows = sorted(set(rng.integers(0, R * Nb, size=48).tolist() + [0, 1023, 1024, R * Nb - 1]))
    compare_attention(wl.scaled(wl.CONFIGS[2], dtype=dtype), o, g, q, rows=rows)
    # finish a scattered set (early stop cascades at 2 completions), prune by threshold, append, compare again
    fin = rng.choice(R * Nb, size=R // 2, replace=False)
    sc = rng.random(R * Nb).astype(np.float32)
    for e in (o, g):
        assert e.finish(fin) == orc.OK
    assert_state_equal(o.state(), g.state())
    nA = int(o.state()["n_active"][0])
    for e in (o, g):
        assert e.prune(orc.THRESHOLD, sc[:nA], threshold=np.full(R, 0.4, np.float32),
                       max_pruned=np.full(R, Nb - 1, np.int32)) == orc.OK
    st = g.state()
    assert_state_equal(o.state(), st)
    check_invariants(st, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
    nA = int(st["n_active"][0])
    assert nA > 1024 or R * Nb < 3000
    k, v = draw(nA, Hkv), draw(nA, Hkv)
    for e in (o, g):
        assert e.append(orc.SEQ_BRANCH, None, None, k, v) == orc.OK
    assert_state_equal(o.state(), g.state())
    act = st["active_handles"][:nA]
    rows = sorted(set(rng.integers(0, nA, size=48).tolist() + [0, nA - 1]))
    compare_attention(wl.scaled(wl.CONFIGS[2], dtype=dtype), o, g, q, rows=rows)


def test_decode_is_deterministic_and_leaves_inputs_alone():
    """Two identical calls give bit-identical outputs (fixed partition, fixed merge order)."""
    import torch
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=4, nb=8, prompt_len=200, length_params=(300, 0.8), length_cap=2000)
    L = wl.lengths(cfg)
    g = GpuEngine(**dims(cfg, wl.pages_needed(cfg, L) + 4, 130))
    populate(cfg, [g], L)
    q = g.c._dev(wl.query(cfg, 0), (cfg.n_q_heads, cfg.head_dim))
    q0 = q.clone()
    a = g.c.decode_attention(q).clone()
    b = g.c.decode_attention(q)
    assert torch.equal(a, b) and torch.equal(q, q0)
    st1 = g.state()
    g.c.decode_attention(q)
    assert_state_equal(st1, g.state())          # attention never changes the integer state


@pytest.mark.parametrize("mode", ["mfma16-per-branch", "mfma16-shared-rows", "natural"])
def test_rows_addressed_by_handle(mode):
    """sart_append_active_by_handle / sart_decode_attention_by_handle against the oracle after the batch was
    thinned (so active order and handle order differ): the appended token lands in the same place as through
    the list form (whole integer state equal, attention equal), output rows of active branches match the
    oracle, every other row of `out` is left alone; both merge forms, several launch shapes."""
    import torch
    natural = mode == "natural"
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=4, nb=6, prompt_len=100, length_params=(200, 0.8), length_cap=1500)
    L = wl.lengths(cfg)
    L[1, 2], L[2, 0] = 16, 31
    pages = wl.pages_needed(cfg, L) + 40
    o, g = _pair(cfg, pages, int(-(-L.max() // 16)) + 2, free_order=wl.free_order(cfg, pages), force_natural_layout=natural)
    pmode = {"mfma16-per-branch": 1, "mfma16-shared-rows": 2, "natural": 1}[mode]
    g.c.set_decode_launch(prompt_mode=pmode)
    populate(cfg, [o, g], L)
    sc = wl.scores(cfg, 0)
    st = o.state()
    act = st["active_handles"][:int(st["n_active"][0])]
    assert o.prune(orc.DROP_LOWEST_K, sc[act], k=2) == orc.OK and g.prune(orc.DROP_LOWEST_K, sc[act], k=2) == orc.OK
    st = o.state()
    act = st["active_handles"][:int(st["n_active"][0])]
    assert o.finish([act[0], act[5]]) == orc.OK and g.finish([act[0], act[5]]) == orc.OK
    H = cfg.n_handles
    for step in (1, 2):
        K, V = wl.step_kv(cfg, step)
        st = o.state()
        act = st["active_handles"][:int(st["n_active"][0])]
        assert o.append(orc.SEQ_BRANCH, None, None, K[act], V[act]) == orc.OK
        g.c.append_active_by_handle(K, V)
        assert_state_equal(o.state(), g.state())
        q = wl.query(cfg, step)
        ref = o.attention(q[act])
        qd = g.c._dev(q, (cfg.n_q_heads, cfg.head_dim))
        for n_wg, skew in ((0, 80), (3, 45), (64, 300)):
            g.c.set_decode_launch(n_wg, pmode, skew)
            for in_kernel in (False, True):
                g.c.set_merge_mode(in_kernel)
                out = torch.full((H, cfg.n_q_heads, cfg.head_dim), -7.5, dtype=torch.float32, device="cuda")
                g.c.decode_attention_by_handle(qd, out)
                got = out.cpu().numpy()
                assert g.c.sync_status() == 0
                assert float(np.abs(got[act].astype(np.float64) - ref).max()) <= TOL["bf16"]
                assert np.all(got[np.setdiff1d(np.arange(H), act)] == -7.5)
                same = g.c.decode_attention(qd[torch.as_tensor(act, device="cuda").long()]).cpu().numpy()
                assert np.array_equal(same, got[act])           # the list form computes the same bits
        g.c.set_merge_mode(False)
        g.c.set_decode_launch(prompt_mode=pmode)
    assert g.c.active_count_hint() == int(o.state()["n_active"][0])


# ---------------------------------------------------------------------------
# waiting branches (Algorithm 1's branch queue): created WAITING, started one by one
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,pt,d", [("f32", 4, 8), ("bf16", 16, 64)])
def test_random_op_sequences_with_waiting_branches(dtype, pt, d):
    """Random prefix / start / split / append / prune / finish sequences on caches whose branches are created
    WAITING (errors included): status and the whole integer state agree with the oracle after every call, and
    the attention of every fifth state and of the final one too (split branches read shared and copied pages)."""
    rng = np.random.default_rng(77)
    R, Nb, num_pages, max_bp, max_pp = 6, 4, 140, 6, 3
    npd = np.float32 if dtype == "f32" else np.uint16
    splits_done = 0
    for trial in range(6):
        kw = dict(n_q_heads=2, n_kv_heads=1, head_dim=d, page_tokens=pt, num_pages=num_pages, max_requests=R,
                  branches_per_request=Nb, finish_quota=int(rng.integers(0, 4)), max_pages_per_branch=max_bp,
                  max_prefix_pages=max_pp, dtype=dtype, start_waiting=True)
        fo = rng.permutation(num_pages).astype(np.int32) if trial % 2 else None
        o, g = orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)

        def draw(n):
            x = rng.standard_normal((n, 1, d)).astype(np.float32)
            return x if dtype == "f32" else wl.f32_to_bf16_bits(x)
        next_req = 0
        for step in range(60):
            st = o.state()
            nA = int(st["n_active"][0])
            waiting = np.flatnonzero(st["branch_state"] == orc.WAITING)
            op = int(rng.integers(0, 10))
            if op in (8, 9) and len(waiting) and nA:
                # splits: waiting branches continue active branches of their request (sometimes a wrong pair)
                act = st["active_handles"][:nA]
                src, dst = [], []
                for b in rng.permutation(waiting)[:int(rng.integers(1, 4))]:
                    cand = act[act // Nb == b // Nb] if rng.random() < 0.9 else act
                    if len(cand):
                        src.append(int(rng.choice(cand))); dst.append(int(b))
                if not src:
                    continue
                if rng.random() < 0.1:
                    dst[0] = int(rng.choice(act))                                     # not waiting
                rc = [e.fork(src, dst) for e in (o, g)]
                splits_done += rc[0] == orc.OK
            elif op == 0 and next_req < R:
                n = int(rng.integers(1, max_pp * pt + 1))
                k, v = draw(n), draw(n)
                rc = [e.append(orc.SEQ_PREFIX, [next_req], [n], k, v) for e in (o, g)]
                next_req += 1
            elif op in (1, 2, 3) and len(waiting):
                m = int(rng.integers(1, min(len(waiting), 5) + 1))
                pool = waiting if rng.random() < 0.85 else np.arange(R * Nb)      # sometimes a branch that is not waiting
                hs = rng.choice(pool, size=min(m, len(pool)), replace=False)
                rc = [e.start(hs) for e in (o, g)]
            elif op in (4, 5) and nA:
                n = rng.integers(0, 2 * pt, size=nA)
                k, v = draw(int(n.sum())), draw(int(n.sum()))
                rc = [e.append(orc.SEQ_BRANCH, None, n, k, v) for e in (o, g)]
            elif op == 6 and nA:
                sc = rng.random(nA).astype(np.float32)
                kwp = dict(k=int(rng.integers(0, 3)), threshold=rng.random(R).astype(np.float32),
                           max_pruned=rng.integers(0, Nb + 1, size=R))
                mode = int(rng.integers(0, 3))
                rc = [e.prune(mode, sc, **kwp) for e in (o, g)]
            elif op == 7 and nA:
                hs = rng.choice(st["active_handles"][:nA], size=int(rng.integers(1, min(nA, 3) + 1)), replace=False)
                rc = [e.finish(hs) for e in (o, g)]
            else:
                continue
            assert rc[0] == rc[1], (trial, step, op, rc)
            so, sg = o.state(), g.state()
            assert_state_equal(so, sg)
            check_invariants(sg, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
            if step % 5 == 4 and int(so["n_active"][0]):
                q = draw(R * Nb).reshape(R * Nb, 1, d).repeat(2, axis=1)
                compare_attention(wl.scaled(wl.CONFIGS[2], dtype=dtype), o, g, q)
        nA = int(o.state()["n_active"][0])
        if nA:
            q = draw(R * Nb).reshape(R * Nb, 1, d).repeat(2, axis=1)
            compare_attention(wl.scaled(wl.CONFIGS[2], dtype=dtype), o, g, q)
    assert splits_done >= 3, splits_done


def test_split_branches_at_the_7b_like_shape():
    """Tree search at a real head geometry: 6 requests x 8 branches, prompts of 300 tokens; one branch per request
    runs 1000+ tokens, splits into three, those run on and split again until all 8 exist; branches are pruned and
    finished along the way.  Whole integer state and every row's attention against the oracle after each phase;
    two layers (the copy of a partly filled page must reach every layer)."""
    rng = np.random.default_rng(21)
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=6, nb=8, prompt_len=300, quota=8)
    R, Nb, pt = cfg.n_requests, cfg.nb, 16
    num_pages, max_bp = 1400, 100
    kw = dims(cfg, num_pages, max_bp)
    fo = wl.free_order(cfg, num_pages)
    o0, o1 = orc.OracleCache(free_order=fo, start_waiting=True, **kw), orc.OracleCache(free_order=fo, start_waiting=True, **kw)
    g = GpuEngine(free_order=fo, start_waiting=True, n_layers=2, **kw)

    def bits(shape):
        return wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))

    def both_layers(fn_oracle, fn_gpu):
        for o in (o0, o1):
            assert fn_oracle(o) == orc.OK
        assert fn_gpu() == orc.OK

    def append(kind, ids, ns):
        n = int(np.sum(ns))
        k0, v0, k1, v1 = (bits((n, cfg.n_kv_heads, cfg.head_dim)) for _ in range(4))
        assert o0.append(kind, ids, ns, k0, v0) == orc.OK and o1.append(kind, ids, ns, k1, v1) == orc.OK
        assert g.c.append_tokens(kind, ids, ns, k0, v0, status=True) == orc.OK
        assert g.c.append_tokens(kind, ids, ns, k1, v1, status=True, layer=1) == orc.OK

    def check():
        so = o0.state()
        assert_state_equal(so, o1.state())
        assert_state_equal(so, g.state())
        check_invariants(so, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
        nA = int(so["n_active"][0])
        act = so["active_handles"][:nA]
        q = bits((nA, cfg.n_q_heads, cfg.head_dim))
        worst = 0.0
        for layer, o in enumerate((o0, o1)):
            got = g.c.decode_attention(q, layer=layer).cpu().numpy().astype(np.float64)
            worst = max(worst, float(np.abs(got - o.attention(q)).max()))
        assert g.c.sync_status() == 0 and worst <= TOL["bf16"], worst
        return act, worst

    for r in range(R):
        append(orc.SEQ_PREFIX, [r], [cfg.prompt_len])
    roots = [r * Nb for r in range(R)]
    both_layers(lambda o: o.start(roots), lambda: g.start(roots))
    append(orc.SEQ_BRANCH, roots, [int(x) for x in rng.integers(1000, 1100, size=R)])        # some end mid-page, some not
    src = [r * Nb for r in range(R) for _ in range(3)]
    dst = [r * Nb + j for r in range(R) for j in (1, 2, 3)]
    both_layers(lambda o: o.fork(src, dst), lambda: g.fork(src, dst))
    act, w1 = check()
    assert len(act) == 4 * R
    append(orc.SEQ_BRANCH, None, [int(x) for x in rng.integers(0, 40, size=len(act))])
    # second generation: branches 1 and 3 of every request split (1 twice)
    src = [r * Nb + j for r in range(R) for j in (1, 1, 3, 2)]
    dst = [r * Nb + j for r in range(R) for j in (4, 5, 6, 7)]
    both_layers(lambda o: o.fork(src, dst), lambda: g.fork(src, dst))
    act, w2 = check()
    assert len(act) == 8 * R
    append(orc.SEQ_BRANCH, None, [int(x) for x in rng.integers(1, 30, size=len(act))])
    check()
    sc = rng.random(len(act)).astype(np.float32)
    both_layers(lambda o: o.prune(orc.DROP_LOWEST_K, sc, k=3), lambda: g.prune(orc.DROP_LOWEST_K, sc, k=3))
    act, _ = check()
    fin = [int(b) for b in act[::3]]
    both_layers(lambda o: o.finish(fin), lambda: g.finish(fin))
    act, w3 = check()
    held = o0.state()["block_tables"][:len(act)].ravel()
    assert np.unique(held[held >= 0], return_counts=True)[1].max() > 1, "no page is shared any more: the case lost its point"
    rest = [int(b) for b in act]
    both_layers(lambda o: o.finish(rest), lambda: g.finish(rest))
    st = g.state()
    assert_state_equal(o0.state(), st)
    assert int(st["free_top"][0]) == num_pages
    print(f"split branches: max abs attention err {max(w1, w2, w3):.3g}")


def test_starting_branches_among_thousands_of_rows():
    """The start plan's scans run over more than one chunk of 1024 rows: 700 requests x 4 branches, started in
    three calls that interleave requests with and without rows already in the batch."""
    rng = np.random.default_rng(5)
    R, Nb, d, pt = 700, 4, 64, 16
    num_pages = R * Nb * 2 + R + 64
    kw = dict(n_q_heads=4, n_kv_heads=2, head_dim=d, page_tokens=pt, num_pages=num_pages, max_requests=R,
              branches_per_request=Nb, finish_quota=2, max_pages_per_branch=3, max_prefix_pages=1, dtype="bf16",
              start_waiting=True)
    o, g = orc.OracleCache(**kw), GpuEngine(**kw)

    def draw(n, heads):
        return wl.f32_to_bf16_bits(rng.standard_normal((n, heads, d)).astype(np.float32))
    for r0 in range(0, R, 100):
        ids = np.arange(r0, min(R, r0 + 100))
        P = rng.integers(1, pt + 1, size=len(ids))
        k, v = draw(int(P.sum()), 2), draw(int(P.sum()), 2)
        for e in (o, g):
            assert e.append(orc.SEQ_PREFIX, ids, P, k, v) == orc.OK
    order = rng.permutation(R * Nb)
    for part in (order[:1100], order[1100:2300], order[2300:]):
        for e in (o, g):
            assert e.start(part) == orc.OK
        assert_state_equal(o.state(), g.state())
        nA = int(o.state()["n_active"][0])
        L = rng.integers(0, 2 * pt, size=nA)
        k, v = draw(int(L.sum()), 2), draw(int(L.sum()), 2)
        for e in (o, g):
            assert e.append(orc.SEQ_BRANCH, None, L % (pt // 2 + 1), k[:int((L % (pt // 2 + 1)).sum())], v[:int((L % (pt // 2 + 1)).sum())]) == orc.OK
        assert_state_equal(o.state(), g.state())
    st = g.state()
    check_invariants(st, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
    nA = int(st["n_active"][0])
    assert nA == R * Nb
    q = draw(R * Nb, 4)
    rows = sorted(set(rng.integers(0, nA, size=40).tolist() + [0, 1023, 1024, 2047, 2048, nA - 1]))
    compare_attention(wl.scaled(wl.CONFIGS[2], dtype="bf16"), o, g, q, rows=rows)
