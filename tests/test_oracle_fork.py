"""Pins of the oracle's branch split (orc_fork) against things other than itself.

The paper's own method never splits a branch; tree search over reasoning
trajectories (Section 2; the Rebase baseline of Section 5.1) does, and what a
split must mean for the KV cache follows from Section 4's rule for the prompt:
what two branches have in common is kept once and released when the last of
them has ended.  Pinned here:
  * a dense shadow that knows nothing of pages: after any sequence of appends,
    splits, finishes and prunes every active branch attends to exactly the
    tokens of its own history (its ancestors' tokens up to each split, then its
    own), by brute force in numpy;
  * page accounting: free + distinct branch pages + prompt pages = all pages
    after every call, shared pages sit at equal logical indices with everything
    before them shared too, and a twin cache that copies instead of sharing
    holds the same lengths, order and attention with more pages in use;
  * the hand-worked trace in tests/golden (release order of shared pages) runs
    in test_oracle_bookkeeping.py.
"""
import numpy as np
import pytest

import oracle as orc
from dense_ref import dense_attention
from helpers import DenseShadow, check_invariants, make_oracle


def _tokens(rng, n, Hkv, d):
    return rng.standard_normal((n, Hkv, d)).astype(np.float32)


class _History:
    """Dense per-branch token history: a split copies the parent's arrays."""

    def __init__(self, Hkv, d):
        self.sh = DenseShadow(Hkv, d)

    def fork(self, src, dst):
        if src in self.sh.private:
            k, v = self.sh.private[src]
            self.sh.private[dst] = (k.copy(), v.copy())
        else:
            self.sh.private.pop(dst, None)


@pytest.mark.parametrize("pt,L0", [(4, 6), (4, 8), (16, 1), (16, 33), (4, 0)])
def test_split_branches_attend_to_their_own_history(pt, L0):
    """One request: branch 0 gets L0 tokens (a partly filled, a full, a single-token last page, no tokens),
    splits into 1 and 2, all three go on with different tokens, 1 splits again into 3."""
    rng = np.random.default_rng(7 + pt + L0)
    Hq, Hkv, d, Nb, P = 4, 2, 8, 4, 5
    o = make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=64, max_req=1, Nb=Nb, max_bp=16, max_pp=4, start_waiting=True)
    hist = _History(Hkv, d)
    k, v = _tokens(rng, P, Hkv, d), _tokens(rng, P, Hkv, d)
    assert o.append(orc.SEQ_PREFIX, [0], [P], k, v) == orc.OK
    hist.sh.add_prefix(0, k, v)
    assert o.start([0]) == orc.OK

    def grow(b, n):
        k, v = _tokens(rng, n, Hkv, d), _tokens(rng, n, Hkv, d)
        assert o.append(orc.SEQ_BRANCH, [b], [n], k, v) == orc.OK
        hist.sh.add_private(b, k, v)

    def check():
        st = o.state()
        nA = int(st["n_active"][0])
        act = st["active_handles"][:nA]
        q = rng.standard_normal((nA, Hq, d)).astype(np.float32)
        out = o.attention(q)
        for a, b in enumerate(act):
            K, V = hist.sh.context(int(b), Nb)
            assert K.shape[0] == P + int(st["seq_lens"][a])
            np.testing.assert_allclose(out[a], dense_attention(q[a].astype(np.float64), K, V), rtol=0, atol=1e-12)
        check_invariants(st, pt=pt, num_pages=64, Nb=Nb, max_req=1)
        return st

    if L0:
        grow(0, L0)
    assert o.fork([0, 0], [1, 2]) == orc.OK
    hist.fork(0, 1); hist.fork(0, 2)
    st = check()
    assert list(st["active_handles"][:3]) == [0, 1, 2] and list(st["seq_lens"][:3]) == [L0] * 3
    full = L0 // pt
    bt = st["block_tables"]
    assert np.array_equal(bt[0][:full], bt[1][:full]) and np.array_equal(bt[0][:full], bt[2][:full])
    if L0 % pt:                                      # the partly filled page was copied, not shared
        assert len({int(bt[0][full]), int(bt[1][full]), int(bt[2][full])}) == 3
    for b, n in ((0, 3), (1, pt + 1), (2, 1)):
        grow(b, n)
    check()
    assert o.fork([1], [3]) == orc.OK
    hist.fork(1, 3)
    grow(3, 2); grow(1, 1)
    st = check()
    used_shared = 64 - int(st["free_top"][0])
    # the parent of the first split ends: its tokens stay readable for the others
    assert o.finish([0]) == orc.OK
    check()
    assert o.prune(orc.DROP_LOWEST_K, np.array([0.3, 0.1, 0.2], np.float32), k=2) == orc.OK
    st = check()
    assert list(st["active_handles"][:1]) == [1]
    assert o.finish([1]) == orc.OK
    st = o.state()
    assert int(st["free_top"][0]) == 64 and sorted(st["free_stack"]) == list(range(64))
    assert used_shared > 0


def test_fork_errors_change_nothing():
    o = make_oracle(pt=4, num_pages=6, max_req=2, Nb=3, max_bp=4, max_pp=1, start_waiting=True)
    one = np.ones((3, 1, 64), np.float32)
    assert o.append(orc.SEQ_PREFIX, [0], [3], one, one) == orc.OK
    assert o.append(orc.SEQ_PREFIX, [1], [3], one, one) == orc.OK
    assert o.start([0, 3]) == orc.OK
    assert o.append(orc.SEQ_BRANCH, [0, 3], [5, 5], np.ones((10, 1, 64), np.float32), np.ones((10, 1, 64), np.float32)) == orc.OK
    before = o.state()
    assert int(before["free_top"][0]) == 0                            # 2 prompt pages + 2 x 2 branch pages: pool exhausted
    for src, dst, want in (([0], [4], orc.E_INVALID),                 # another request's branch
                           ([0], [9], orc.E_INVALID), ([-1], [1], orc.E_INVALID),
                           ([0, 0], [1, 1], orc.E_INVALID),           # a branch cannot start twice
                           ([1], [2], orc.E_STATE),                   # the source is not in the batch
                           ([0], [3], orc.E_INVALID),
                           ([3], [3], orc.E_STATE),                   # the destination is not waiting
                           ([0], [1], orc.E_OOM_PAGES)):              # no page for the copy of the partly filled page
        assert o.fork(src, dst) == want, (src, dst)
        after = o.state()
        for key in before:
            np.testing.assert_array_equal(before[key], after[key], err_msg=key)


@pytest.mark.parametrize("seed", range(6))
def test_random_ops_with_splits_against_a_copying_twin(seed):
    """Random appends, splits, finishes and prunes on two caches: one shares pages on a split, its twin starts
    the new branch empty and appends the parent's tokens again.  Same batch order, lengths and attention after
    every call; the sharing cache never uses more pages; invariants hold throughout."""
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv, d, pt, Nb, R, P = 2, 1, 8, 4, 5, 2, 3
    num_pages = 400
    mk = lambda: make_oracle(Hq=Hq, Hkv=Hkv, d=d, pt=pt, num_pages=num_pages, max_req=R, Nb=Nb, Q=3, max_bp=40, max_pp=2,
                             start_waiting=True)
    a, b = mk(), mk()
    toks = {}                                       # handle -> (K, V) float32 history (what the twin re-appends)
    for r in range(R):
        k, v = _tokens(rng, P, Hkv, d), _tokens(rng, P, Hkv, d)
        for o in (a, b):
            assert o.append(orc.SEQ_PREFIX, [r], [P], k, v) == orc.OK
        for o in (a, b):
            assert o.start([r * Nb]) == orc.OK
        toks[r * Nb] = (np.zeros((0, Hkv, d), np.float32), np.zeros((0, Hkv, d), np.float32))
    saved = 0
    for step in range(60):
        st = a.state()
        nA = int(st["n_active"][0])
        if nA == 0:
            break
        act = [int(x) for x in st["active_handles"][:nA]]
        waiting = [h for h in range(R * Nb) if st["branch_state"][h] == orc.WAITING]
        op = ("grow", "fork")[step] if step < 2 else rng.choice(["grow", "grow", "fork", "finish", "prune"])
        if op == "grow":
            n = [int(x) for x in rng.integers(pt if step == 0 else 0, 2 * pt, size=nA)]
            k, v = _tokens(rng, sum(n), Hkv, d), _tokens(rng, sum(n), Hkv, d)
            for o in (a, b):
                assert o.append(orc.SEQ_BRANCH, None, n, k, v) == orc.OK
            off = 0
            for h, c in zip(act, n):
                toks[h] = (np.concatenate([toks[h][0], k[off:off + c]]), np.concatenate([toks[h][1], v[off:off + c]]))
                off += c
        elif op == "fork" and waiting:
            pairs = []
            for dst in waiting:
                srcs = [h for h in act if h // Nb == dst // Nb]
                if srcs and (step < 2 or rng.random() < 0.6):
                    pairs.append((int(rng.choice(srcs)), dst))
            if not pairs:
                continue
            src, dst = [p[0] for p in pairs], [p[1] for p in pairs]
            assert a.fork(src, dst) == orc.OK
            assert b.start(dst) == orc.OK
            n = [len(toks[s][0]) for s in src]
            if sum(n):
                assert b.append(orc.SEQ_BRANCH, dst, n, np.concatenate([toks[s][0] for s in src]),
                                np.concatenate([toks[s][1] for s in src])) == orc.OK
            for s, t in pairs:
                toks[t] = toks[s]
        elif op == "finish":
            fin = [h for h in act if rng.random() < 0.15]
            for o in (a, b):
                assert o.finish(fin) == orc.OK
        elif op == "prune":
            sc = rng.random(nA).astype(np.float32)
            for o in (a, b):
                assert o.prune(orc.DROP_LOWEST_K, sc, k=1) == orc.OK
        sa, sb = a.state(), b.state()
        for key in ("n_active", "active_handles", "seq_lens", "branch_state", "req_counters", "prefix_refcnt"):
            np.testing.assert_array_equal(sa[key], sb[key], err_msg=f"{key} after step {step} ({op})")
        check_invariants(sa, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
        check_invariants(sb, pt=pt, num_pages=num_pages, Nb=Nb, max_req=R)
        assert sa["free_top"][0] >= sb["free_top"][0]
        saved = max(saved, int(sa["free_top"][0] - sb["free_top"][0]))
        n2 = int(sa["n_active"][0])
        if n2:
            q = rng.standard_normal((n2, Hq, d)).astype(np.float32)
            np.testing.assert_allclose(a.attention(q), b.attention(q), rtol=0, atol=1e-13)
    assert saved > 0, "no split ever shared a page"
