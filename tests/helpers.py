"""Shared test helpers: a dense shadow record of what was appended, and the
page-accounting invariants (these hold for any correct implementation, so the
same checks run on the oracle's state and on the HIP library's state)."""
import numpy as np

import oracle as orc


def make_oracle(*, Hq=4, Hkv=1, d=64, pt=16, num_pages=64, max_req=2, Nb=4, Q=0, max_bp=32, max_pp=16,
                dtype="f32", free_order=None, start_waiting=False):
    return orc.OracleCache(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, page_tokens=pt, num_pages=num_pages,
                           max_requests=max_req, branches_per_request=Nb, finish_quota=Q,
                           max_pages_per_branch=max_bp, max_prefix_pages=max_pp, dtype=dtype,
                           free_order=free_order, start_waiting=start_waiting)


class DenseShadow:
    """Keeps every appended token in dense per-sequence float64 arrays."""

    def __init__(self, Hkv, d):
        self.Hkv, self.d = Hkv, d
        self.prefix = {}   # request -> (K [T,Hkv,d], V)
        self.private = {}  # handle  -> (K, V)

    def _cat(self, store, key, k, v):
        k = np.asarray(k, np.float64).reshape(-1, self.Hkv, self.d)
        v = np.asarray(v, np.float64).reshape(-1, self.Hkv, self.d)
        if key in store:
            store[key] = (np.concatenate([store[key][0], k]), np.concatenate([store[key][1], v]))
        else:
            store[key] = (k, v)

    def add_prefix(self, r, k, v):
        self._cat(self.prefix, r, k, v)

    def add_private(self, b, k, v):
        self._cat(self.private, b, k, v)

    def context(self, b, Nb):
        r = b // Nb
        empty = np.zeros((0, self.Hkv, self.d))
        pk, pv = self.prefix.get(r, (empty, empty))
        bk, bv = self.private.get(b, (empty, empty))
        return np.concatenate([pk, bk]), np.concatenate([pv, bv])


def check_invariants(st, *, pt, num_pages, Nb, max_req):
    """Page conservation and reference counts (spec invariant):
    free + private pages of active branches + prefix pages of live requests ==
    num_pages, no page listed twice - except that branches of one request may hold a page together after a
    fork, then at the same logical index and with every earlier page shared too -, refcnt[r] == number of
    active and waiting branches."""
    nA = int(st["n_active"][0])
    top = int(st["free_top"][0])
    pages = list(st["free_stack"][:top])
    assert all(p >= 0 for p in pages)
    assert np.all(st["free_stack"][top:] == -1)
    assert np.all(st["active_handles"][nA:] == -1)
    assert np.all(st["seq_lens"][nA:] == 0)
    assert np.all(st["block_tables"][nA:] == -1)
    live = np.zeros(max_req, np.int64)
    holders = {}                                  # branch page -> (logical index, request, rows holding it)
    for a in range(nA):
        b = int(st["active_handles"][a])
        assert st["branch_state"][b] == orc.ACTIVE
        live[b // Nb] += 1
        n = -(-int(st["seq_lens"][a]) // pt)
        row = st["block_tables"][a]
        assert np.all(row[:n] >= 0) and np.all(row[n:] == -1), (a, n, row)
        for l in range(n):
            pg = int(row[l])
            if pg in holders:
                l0, r0, rows0 = holders[pg]
                assert (l0, r0) == (l, b // Nb), f"page {pg} shared at different places"
                for a0 in rows0:                  # who shares page l shares what comes before it
                    assert np.array_equal(st["block_tables"][a0][:l], row[:l])
                rows0.append(a)
            else:
                holders[pg] = (l, b // Nb, [a])
                pages.append(pg)
    assert len(set(int(h) for h in st["active_handles"][:nA])) == nA
    assert np.sum(st["branch_state"] == orc.ACTIVE) == nA
    waiting = (st["branch_state"] == orc.WAITING).reshape(max_req, Nb).sum(axis=1)
    live = live + waiting                     # awaiting branches hold the prompt too
    np.testing.assert_array_equal(st["prefix_refcnt"], live)
    for r in range(max_req):
        n = -(-int(st["prefix_lens"][r]) // pt)
        row = st["prefix_tables"][r]
        if live[r] > 0:
            assert np.all(row[:n] >= 0) and np.all(row[n:] == -1)
            pages += list(row[:n])
        else:
            assert np.all(row == -1), (r, row)
    assert len(pages) == num_pages, (len(pages), num_pages)
    assert sorted(int(p) for p in pages) == list(range(num_pages))


def assert_state_equal(a, b):
    for key in a:
        np.testing.assert_array_equal(a[key], b[key], err_msg=key)


# ---------------------------------------------------------------------------
# golden trace runner (tests/golden/bookkeeping_small.json).  `engine` needs
# append(kind, ids, n_tokens, k, v) -> status, prune(...) -> status,
# finish(handles) -> status, state() -> dict; `done(r)` is optional.
# ---------------------------------------------------------------------------
def run_golden_scenario(scn, engine, Hkv, d, np_dtype, done=None):
    desc = scn["desc"]
    for i, step in enumerate(scn["steps"]):
        op = step["op"]
        if op in ("prefix", "branch"):
            kind = orc.SEQ_PREFIX if op == "prefix" else orc.SEQ_BRANCH
            ids, n = step["ids"], step["n"]
            if n is not None:
                total = int(np.sum(n))
            elif ids is not None:
                total = len(ids)
            else:
                total = int(engine.state()["n_active"][0])
            kv = np.ones((total, Hkv, d), np_dtype)
            rc = engine.append(kind, ids, n, kv, kv)
        elif op == "prune":
            rc = engine.prune(step["mode"], np.asarray(step["scores"], np.float32), k=step.get("k", 0),
                              threshold=step.get("threshold"), max_pruned=step.get("max_pruned"))
        elif op == "finish":
            rc = engine.finish(step["handles"])
        elif op == "start":
            rc = engine.start(step["handles"])
        elif op == "fork":
            rc = engine.fork(step["src"], step["dst"])
        else:
            raise ValueError(op)
        assert rc == step["status"], (scn["name"], i, op, rc)
        st = engine.state()
        check_invariants(st, pt=desc["pt"], num_pages=desc["num_pages"], Nb=desc["Nb"], max_req=desc["max_req"])
        exp = step["expect"]
        nA = int(st["n_active"][0])
        where = f"{scn['name']} step {i} ({op})"
        if "active" in exp:
            assert list(st["active_handles"][:nA]) == exp["active"], where
        if "seq_lens" in exp:
            assert list(st["seq_lens"][:nA]) == exp["seq_lens"], where
        if "free_stack" in exp:
            assert list(st["free_stack"][:int(st["free_top"][0])]) == exp["free_stack"], where
        if "block_tables" in exp:
            assert st["block_tables"][:nA].tolist() == exp["block_tables"], where
        if "prefix_tables" in exp:
            assert st["prefix_tables"].tolist() == exp["prefix_tables"], where
        if "refcnt" in exp:
            assert list(st["prefix_refcnt"]) == exp["refcnt"], where
        if "branch_state" in exp:
            assert list(st["branch_state"]) == exp["branch_state"], where
        if "counters" in exp:
            assert st["req_counters"].tolist() == exp["counters"], where
        if "done" in exp and done is not None:
            assert [bool(done(r)) for r in range(desc["max_req"])] == exp["done"], where
