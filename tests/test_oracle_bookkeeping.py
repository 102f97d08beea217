"""Pins of the oracle's bookkeeping: hand-worked traces, conservation,
policy algebra, Algorithm 1's termination test and survivors unchanged."""
import json
import os

import numpy as np
import pytest

import oracle as orc
from helpers import assert_state_equal, check_invariants, make_oracle, run_golden_scenario

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bookkeeping_small.json")
with open(GOLDEN) as f:
    SCENARIOS = json.load(f)["scenarios"]


@pytest.mark.parametrize("scn", SCENARIOS, ids=[s["name"] for s in SCENARIOS])
def test_hand_worked_traces(scn):
    d = scn["desc"]
    o = make_oracle(Hq=2, Hkv=1, d=8, pt=d["pt"], num_pages=d["num_pages"], max_req=d["max_req"], Nb=d["Nb"],
                    Q=d["Q"], max_bp=d["max_bp"], max_pp=d["max_pp"], start_waiting=d.get("start_waiting", False))
    run_golden_scenario(scn, o, 1, 8, np.float32, done=o.request_done)


def _populated(rng, *, R=3, Nb=4, Q=0, pt=4, num_pages=200, maxL=30, P=6, free_order=None):
    o = make_oracle(Hq=2, Hkv=1, d=8, pt=pt, num_pages=num_pages, max_req=R, Nb=Nb, Q=Q, max_bp=16, max_pp=4,
                    free_order=free_order)
    one = lambda n: np.ones((n, 1, 8), np.float32)
    for r in range(R):
        assert o.append(orc.SEQ_PREFIX, [r], [P], one(P), one(P)) == orc.OK
    L = rng.integers(1, maxL, size=R * Nb)
    assert o.append(orc.SEQ_BRANCH, None, L, one(L.sum()), one(L.sum())) == orc.OK
    return o, L


def test_P5_conservation_under_random_ops():
    """Random append / prune / finish sequences keep every page accounted for."""
    rng = np.random.default_rng(55)
    for trial in range(20):
        R, Nb, pt, num_pages = 4, 4, 4, 150
        o, _ = _populated(rng, R=R, Nb=Nb, Q=int(rng.integers(0, 4)), pt=pt, num_pages=num_pages)
        for _ in range(30):
            st = o.state()
            nA = int(st["n_active"][0])
            check_invariants(st, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
            if nA == 0:
                break
            op = rng.integers(0, 4)
            if op == 0:
                n = rng.integers(0, 6, size=nA)
                kv = np.ones((int(n.sum()), 1, 8), np.float32)
                assert o.append(orc.SEQ_BRANCH, None, n, kv, kv) in (orc.OK, orc.E_OOM_PAGES, orc.E_INVALID)
            elif op == 1:
                mode = int(rng.integers(0, 3))
                sc = rng.random(nA).astype(np.float32)
                assert o.prune(mode, sc, k=int(rng.integers(0, 3)), threshold=rng.random(R).astype(np.float32),
                               max_pruned=rng.integers(0, Nb, size=R)) == orc.OK
            else:
                hs = rng.choice(st["active_handles"][:nA], size=min(nA, int(rng.integers(1, 3))), replace=False)
                assert o.finish(hs) == orc.OK
        # terminate everything: the stack must hold every page again
        st = o.state()
        nA = int(st["n_active"][0])
        if nA:
            assert o.prune(orc.KEEP_TOP_K, np.zeros(nA, np.float32), k=0) == orc.OK
        st = o.state()
        assert st["free_top"][0] == num_pages and st["n_active"][0] == 0
        check_invariants(st, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)


def test_P10_policy_algebra():
    rng = np.random.default_rng(10)
    for trial in range(10):
        seed = int(rng.integers(1 << 30))
        Nb = 6
        sc = np.random.default_rng(seed).random(3 * Nb).astype(np.float32)
        sc[rng.integers(0, 3 * Nb, size=4)] = 0.25  # ties
        for k in range(0, Nb + 2):
            a, _ = _populated(np.random.default_rng(seed), R=3, Nb=Nb)
            b, _ = _populated(np.random.default_rng(seed), R=3, Nb=Nb)
            assert a.prune(orc.KEEP_TOP_K, sc, k=k) == orc.OK
            assert b.prune(orc.DROP_LOWEST_K, sc, k=max(0, Nb - k)) == orc.OK
            assert_state_equal(a.state(), b.state())
            assert a.state()["n_active"][0] == 3 * min(k, Nb)
    # threshold = +inf with cap Nb prunes all; -inf prunes none
    o, _ = _populated(rng, R=2, Nb=4)
    before = o.state()
    assert o.prune(orc.THRESHOLD, rng.random(8).astype(np.float32), threshold=[-np.inf] * 2, max_pruned=[4, 4]) == orc.OK
    assert_state_equal(before, o.state())
    assert o.prune(orc.THRESHOLD, rng.random(8).astype(np.float32), threshold=[np.inf] * 2, max_pruned=[4, 4]) == orc.OK
    assert o.state()["n_active"][0] == 0
    # NaN never pruned, even by +inf threshold; in key modes NaN ranks highest
    o, _ = _populated(rng, R=1, Nb=4)
    sc = np.array([np.nan, 0.3, 0.2, 0.9], np.float32)
    assert o.prune(orc.THRESHOLD, sc, threshold=[np.inf], max_pruned=[4]) == orc.OK
    assert list(o.state()["active_handles"][:1]) == [0]
    o, _ = _populated(rng, R=1, Nb=4)
    assert o.prune(orc.KEEP_TOP_K, sc, k=1) == orc.OK
    assert list(o.state()["active_handles"][:1]) == [0]
    # cap in a key mode keeps the lowest keys as victims
    o, _ = _populated(rng, R=1, Nb=4)
    assert o.prune(orc.DROP_LOWEST_K, np.array([0.4, 0.1, 0.3, 0.2], np.float32), k=3, max_pruned=[2]) == orc.OK
    assert list(o.state()["active_handles"][:2]) == [0, 2]


def test_P11_termination_predicate_matches_algorithm1():
    """done(r) iff completed >= Q or completed + pruned == Nb, checked against
    counts kept by the test itself while branches leave one by one."""
    rng = np.random.default_rng(11)
    for trial in range(30):
        Nb, Q = 6, int(rng.integers(1, 5))
        o, _ = _populated(rng, R=1, Nb=Nb, Q=Q)
        completed = pruned = 0
        alive = list(range(Nb))
        while alive:
            assert o.request_done(0) == (completed >= Q or completed + pruned == Nb)
            b = int(rng.choice(alive))
            if rng.random() < 0.5:
                assert o.finish([b]) == orc.OK
                completed += 1
                alive.remove(b)
                if completed >= Q:   # early stop terminates the rest (not counted as pruned)
                    alive = []
            else:
                st = o.state()
                nA = int(st["n_active"][0])
                sc = np.ones(nA, np.float32)
                sc[list(st["active_handles"][:nA]).index(b)] = 0.0
                assert o.prune(orc.DROP_LOWEST_K, sc, k=1) == orc.OK
                pruned += 1
                alive.remove(b)
            st = o.state()
            assert list(st["req_counters"][0]) == [completed, pruned]
            assert sorted(st["active_handles"][:int(st["n_active"][0])]) == sorted(alive)
        assert o.request_done(0)
        assert o.state()["free_top"][0] == 200


def test_P4_pruning_leaves_survivors_outputs_unchanged():
    rng = np.random.default_rng(4)
    Hq, Hkv, d, pt, R, Nb = 4, 2, 16, 4, 2, 4
    o = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=100, max_req=R, Nb=Nb, max_bp=16, max_pp=4)
    f = lambda n: rng.standard_normal((n, Hkv, d)).astype(np.float32)
    for r in range(R):
        o.append(orc.SEQ_PREFIX, [r], [9], f(9), f(9))
    L = rng.integers(1, 40, size=R * Nb)
    o.append(orc.SEQ_BRANCH, None, L, f(L.sum()), f(L.sum()))
    q = rng.standard_normal((R * Nb, Hq, d)).astype(np.float32)
    before = o.attention(q)
    handles_before = o.state()["active_handles"][:R * Nb].copy()
    assert o.prune(orc.KEEP_TOP_K, rng.random(R * Nb).astype(np.float32), k=2) == orc.OK
    st = o.state()
    nA = int(st["n_active"][0])
    assert nA == 4
    surv = st["active_handles"][:nA]
    rows = [list(handles_before).index(h) for h in surv]
    assert rows == sorted(rows)  # stable compaction
    after = o.attention(q[rows])
    np.testing.assert_array_equal(after, before[rows])
    # new appends reuse freed pages and still do not disturb the others
    o.append(orc.SEQ_BRANCH, [int(surv[0])], [20], f(20), f(20))
    again = o.attention(q[rows])
    np.testing.assert_array_equal(again[1:], before[rows][1:])
    assert np.abs(again[0] - before[rows][0]).max() > 1e-6


def test_argument_errors_change_nothing():
    rng = np.random.default_rng(2)
    o, _ = _populated(rng, R=2, Nb=2)
    s0 = o.state()
    one = np.ones((2, 1, 8), np.float32)
    assert o.append(orc.SEQ_BRANCH, [0, 0], [1, 1], one, one) == orc.E_INVALID      # duplicate
    assert o.append(orc.SEQ_BRANCH, [99], [1], one[:1], one[:1]) == orc.E_INVALID   # range
    assert o.append(orc.SEQ_BRANCH, None, [1, 1], one, one) == orc.E_INVALID        # count != active
    assert o.finish([0, 0]) == orc.E_INVALID
    assert o.finish([-1]) == orc.E_INVALID
    assert o.prune(orc.DROP_LOWEST_K, np.zeros(3, np.float32), k=1) == orc.E_INVALID  # too few scores
    assert o.prune(5, np.zeros(4, np.float32), k=1) == orc.E_INVALID
    assert_state_equal(s0, o.state())
    # a prefix append after a branch append of the same request is refused
    assert o.append(orc.SEQ_PREFIX, [0], [1], one[:1], one[:1]) == orc.E_STATE
    assert_state_equal(s0, o.state())


def test_integer_state_does_not_depend_on_the_head_geometry():
    """The same call sequence on caches that differ only in heads, head size and element type leaves the same
    integer state (the full-size GPU parity tests compare against a one-head, 8-element oracle cache)."""
    rng = np.random.default_rng(91)
    R, Nb, pt, num_pages = 4, 4, 4, 160
    fo = rng.permutation(num_pages).astype(np.int32)
    geoms = [dict(Hq=2, Hkv=1, d=8, dtype="f32"), dict(Hq=12, Hkv=3, d=32, dtype="bf16")]
    caches = [make_oracle(pt=pt, num_pages=num_pages, max_req=R, Nb=Nb, Q=2, max_bp=16, max_pp=4, free_order=fo, **gm)
              for gm in geoms]

    def kv(n, gm):
        return np.zeros((n, gm["Hkv"], gm["d"]), np.float32 if gm["dtype"] == "f32" else np.uint16)

    def all_do(fn):
        rcs = [fn(c, gm) for c, gm in zip(caches, geoms)]
        assert rcs[0] == rcs[1]
        assert_state_equal(caches[0].state(), caches[1].state())
        return rcs[0]

    for r in range(R):
        all_do(lambda c, gm: c.append(orc.SEQ_PREFIX, [r], [5 + r], kv(5 + r, gm), kv(5 + r, gm)))
    for _ in range(40):
        st = caches[0].state()
        nA = int(st["n_active"][0])
        if nA == 0:
            break
        op = int(rng.integers(0, 4))
        if op <= 1:
            n = rng.integers(0, 7, size=nA)
            all_do(lambda c, gm: c.append(orc.SEQ_BRANCH, None, n, kv(int(n.sum()), gm), kv(int(n.sum()), gm)))
        elif op == 2:
            sc = rng.random(nA).astype(np.float32)
            mode, k = int(rng.integers(0, 3)), int(rng.integers(0, 3))
            th, mp = rng.random(R).astype(np.float32), rng.integers(0, Nb, size=R)
            all_do(lambda c, gm: c.prune(mode, sc, k=k, threshold=th, max_pruned=mp))
        else:
            hs = rng.choice(st["active_handles"][:nA], size=1)
            all_do(lambda c, gm: c.finish(hs))
