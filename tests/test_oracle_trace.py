"""Order-statistic pins of the early-stop cascade (Section 3, Lemma 1)."""
from math import comb

import numpy as np

import oracle as orc
from helpers import check_invariants, make_oracle
from oracle.trace import run_trace


def _trace(R, Nb, Q, delta, n_steps, prune_every=0, prune_k=0, scores=None, checks=None):
    pt = 4
    num_pages = R * Nb * (n_steps // pt + 2) + R
    o = make_oracle(Hq=1, Hkv=1, d=8, pt=pt, num_pages=num_pages, max_req=R, Nb=Nb, Q=Q,
                    max_bp=n_steps // pt + 2, max_pp=1)
    one = np.ones((R * Nb, 1, 8), np.float32)
    for r in range(R):
        assert o.append(orc.SEQ_PREFIX, [r], [1], one[:1], one[:1]) == orc.OK
    res = run_trace(o, targets=delta.reshape(-1), step_kv=lambda s: (one, one), n_steps=n_steps,
                    prune_every=prune_every, prune_k=prune_k, scores=scores, on_call=checks)
    return o, res, num_pages


def test_P9_early_stop_step_is_Qth_smallest_length():
    """Without pruning, the decode steps a request needs equal the Q-th smallest
    branch length (Section 3, Solution 1), exactly, per request."""
    rng = np.random.default_rng(9)
    R, Nb, Q = 50, 8, 4
    delta = rng.integers(1, 60, size=(R, Nb))
    o, res, num_pages = _trace(R, Nb, Q, delta, 64)
    expect = np.sort(delta, axis=1)[:, Q - 1]
    np.testing.assert_array_equal(res["done_step"], expect)
    st = o.state()
    assert st["n_active"][0] == 0 and st["free_top"][0] == num_pages
    # completed counts: branches with delta <= the Q-th smallest completed, the rest early-stopped
    for r in range(R):
        n_done = int(np.sum(delta[r] <= expect[r]))
        assert st["req_counters"][r, 0] == n_done
        states = st["branch_state"][r * Nb:(r + 1) * Nb]
        assert np.sum(states == orc.COMPLETED) == n_done
        assert np.sum(states == orc.EARLY_STOPPED) == Nb - n_done


def test_P9_lemma1_cdf():
    """Empirical CDF of the early-stop step over many requests follows Lemma 1:
    F_(M)(x; N) = sum_{i=M..N} C(N,i) F(x)^i (1-F(x))^(N-i), here with lengths
    uniform on 1..40 so F(x) = x/40."""
    rng = np.random.default_rng(91)
    R, Nb, Q, hi = 3000, 8, 4, 40
    delta = rng.integers(1, hi + 1, size=(R, Nb))
    _, res, _ = _trace(R, Nb, Q, delta, hi)
    xs = np.arange(1, hi + 1)
    emp = np.array([(res["done_step"] <= x).mean() for x in xs])
    F = xs / hi
    lemma = sum(comb(Nb, i) * F ** i * (1 - F) ** (Nb - i) for i in range(Q, Nb + 1))
    assert np.abs(emp - lemma).max() < 0.04  # DKW: P(sup dev > 0.04 | n=3000) < 2e-4
    # and it increases with N at fixed M (the lemma's consequence the paper draws)
    lemma6 = sum(comb(6, i) * F ** i * (1 - F) ** (6 - i) for i in range(Q, 7))
    assert np.all(lemma >= lemma6 - 1e-12)


def test_trace_with_capped_pruning_keeps_invariants():
    rng = np.random.default_rng(92)
    R, Nb, Q = 6, 8, 4
    delta = rng.integers(5, 120, size=(R, Nb))
    sc = lambda e: np.random.default_rng(1000 + e).random(R * Nb).astype(np.float32)
    seen = []

    def checks(name, step, cache, extra):
        st = cache.state()
        check_invariants(st, pt=4, num_pages=cache.num_pages, Nb=Nb, max_req=R)
        seen.append(name)
        # Algorithm 1's caps: never more than beta pruned before a completion, never all branches pruned
        c, p = st["req_counters"][:, 0], st["req_counters"][:, 1]
        assert np.all(p <= np.where(c == 0, Nb // 2, Nb - 1))

    o, res, num_pages = _trace(R, Nb, Q, delta, 128, prune_every=10, prune_k=2, scores=sc, checks=checks)
    assert {"append", "finish", "prune"} <= set(seen)
    assert np.all(res["done_step"] > 0)
    assert o.state()["free_top"][0] == num_pages
