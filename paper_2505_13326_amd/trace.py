"""Host step loop over the HIP library: the decode / maintenance cadence of the
paper's serving loop (Algorithm 1, Decode) with the caller owning the loop.

Per step s = 1..n_steps
    sart_append_tokens   one token of K/V for every active branch
    sart_decode_attention
    sart_finish_branch   the branches whose length reached their target
                         (completed branches leave the batch; once Q of a
                         request's branches completed the rest are early-stopped:
                         Section 3, Solution 1)
    every `prune_every` steps: sart_prune_branches, dropping each request's
                         `prune_k` lowest-scoring branches under Algorithm 1's
                         cap max_num_pruned = Nb/2 before the request's first
                         completion and Nb-1 after it (Section 3, Solution 2).
The loop keeps a host copy of the active list and lengths; it reads the state
back only after a call that changes the batch (finish, prune), so plain decode
steps enqueue without waiting for the device.
"""
from __future__ import annotations

import numpy as np

from .binding import DROP_LOWEST_K, SEQ_BRANCH


def run_trace(cache, *, targets, step_kv, query, n_steps, prune_every=0, prune_k=0, scores=None, out=None,
              on_call=None):
    """cache: SartCache holding the initial state.
    targets: int array by handle, private length at which a branch completes.
    step_kv(s) -> (K, V) device tensors [R*Nb, Hkv, d] by handle; query(s) -> Q device [R*Nb, Hq, d];
    scores(event) -> device float32 [R*Nb] by handle.
    out: optional preallocated float32 device tensor [R*Nb, Hq, d] for the attention output.
    on_call(name, step, cache, extra): hook after every library call (tests).
    Returns dict(branch_steps, active_per_step, done_step)."""
    import torch
    Nb, R = cache.Nb, cache.max_req
    st = cache.get_state(fields=("n_active", "active_handles", "seq_lens", "req_counters"))
    nA = int(st["n_active"][0])
    act = st["active_handles"][:nA].copy()
    lens = np.zeros(R * Nb, np.int64)
    lens[act] = st["seq_lens"][:nA]
    completed = st["req_counters"][:, 0].copy()
    pruned = st["req_counters"][:, 1].copy()
    done_step = np.zeros(R, np.int64)
    quota_on = 1 <= cache.Q <= Nb
    active_per_step = []
    event = 0
    act_dev = torch.from_numpy(act.astype(np.int64)).cuda()

    def refresh():
        nonlocal act, act_dev, completed, pruned
        s = cache.get_state(fields=("n_active", "active_handles", "req_counters"))
        n = int(s["n_active"][0])
        act = s["active_handles"][:n].copy()
        act_dev = torch.from_numpy(act.astype(np.int64)).cuda()
        completed = s["req_counters"][:, 0].copy()
        pruned = s["req_counters"][:, 1].copy()

    for s in range(1, n_steps + 1):
        nA = len(act)
        active_per_step.append(nA)
        if nA == 0:
            continue
        K, V = step_kv(s)
        cache.append_tokens(SEQ_BRANCH, None, None, K[act_dev], V[act_dev])
        lens[act] += 1
        if on_call:
            on_call("append", s, cache, act)
        q = query(s)[act_dev]
        o = cache.decode_attention(q, out=None if out is None else out[:nA])
        if on_call:
            on_call("attention", s, cache, (act, o))
        fin = act[lens[act] == targets[act]]
        if len(fin):
            cache.finish_branch(fin)
            refresh()
            if on_call:
                on_call("finish", s, cache, fin)
        if prune_every and s % prune_every == 0:
            if len(act):
                cap = np.where(completed == 0, Nb // 2, Nb - 1).astype(np.int32)
                cache.prune_branches(DROP_LOWEST_K, scores(event)[act_dev].contiguous(), k=prune_k, max_pruned=cap)
                refresh()
                if on_call:
                    on_call("prune", s, cache, None)
            event += 1
        done = ((completed >= cache.Q) if quota_on else np.zeros(R, bool)) | (completed + pruned == Nb)
        done_step[(done_step == 0) & done] = s
    return {"branch_steps": int(np.sum(active_per_step)), "active_per_step": np.asarray(active_per_step),
            "done_step": done_step}
