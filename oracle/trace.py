"""Decode-loop trace on the oracle cache (TEST INFRASTRUCTURE).

The caller owns the step loop (Algorithm 1 passes T to Decode; here one step
is one token per active branch).  Per step s = 1..n_steps:
    append one token to every active branch            (Section 2: one token per decode step)
    [attention over the active branches]
    finish the branches whose length reached their target
                                                       (Algorithm 1, Decode: completed branches
                                                        removed and counted; Section 3,
                                                        Solution 1: early stop at Q completions)
    every `prune_every` steps: drop each request's `prune_k` lowest-scoring branches, never
    exceeding Algorithm 1's max_num_pruned: beta = Nb/2 while the request has no completion
    (exploration phase), Nb - 1 afterwards (exploitation phase; Section 3, Solution 2).
Shares no code with the HIP library's own step loop.
"""
from __future__ import annotations

import numpy as np

from . import DROP_LOWEST_K, OK, SEQ_BRANCH


def run_trace(cache, *, targets, step_kv, n_steps, prune_every=0, prune_k=0, scores=None, query=None,
              on_call=None):
    """targets: int array by handle, private length at which a branch completes.
    step_kv(s) -> (K, V) by handle; scores(event) -> float32 by handle; query(s) -> Q by handle.
    on_call(name, step, cache, extra) is invoked after every library call.
    Returns dict(done_step[r], branch_steps, active_per_step, outputs (if query))."""
    R, Nb = cache.max_req, cache.Nb
    done_step = np.zeros(R, np.int64)
    active_per_step = []
    outputs = {}
    event = 0
    for s in range(1, n_steps + 1):
        st = cache.state()
        nA = int(st["n_active"][0])
        active_per_step.append(nA)
        if nA == 0:
            continue
        act = st["active_handles"][:nA]
        K, V = step_kv(s)
        rc = cache.append(SEQ_BRANCH, None, None, K[act], V[act])
        assert rc == OK, rc
        if on_call:
            on_call("append", s, cache, act)
        if query is not None:
            outputs[s] = (act.copy(), cache.attention(query(s)[act]))
            if on_call:
                on_call("attention", s, cache, outputs[s])
        lens = st["seq_lens"][:nA] + 1
        fin = act[lens == targets[act]]
        if len(fin):
            assert cache.finish(fin) == OK
            if on_call:
                on_call("finish", s, cache, fin)
        if prune_every and s % prune_every == 0:
            st = cache.state()
            nA = int(st["n_active"][0])
            if nA:
                completed = st["req_counters"][:, 0]
                cap = np.where(completed == 0, Nb // 2, Nb - 1).astype(np.int32)
                sc = scores(event)[st["active_handles"][:nA]]
                assert cache.prune(DROP_LOWEST_K, sc, k=prune_k, max_pruned=cap) == OK
                if on_call:
                    on_call("prune", s, cache, sc)
            event += 1
        for r in range(R):
            if done_step[r] == 0 and cache.request_done(r):
                done_step[r] = s
    return {"done_step": done_step, "branch_steps": int(np.sum(active_per_step)),
            "active_per_step": np.asarray(active_per_step), "outputs": outputs}
