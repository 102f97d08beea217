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


def run_trace_device(cache, *, targets, step_kv, query, n_steps, prune_every=0, prune_k=0, scores=None, out=None,
                     graph=False, poll_every=8, on_step=None):
    """The same loop with the step kept on the device: the host never learns which branches are in the batch.
    Per step sart_append_active_by_handle, sart_decode_attention_by_handle (inputs and output addressed by
    branch handle, so nobody gathers rows) and sart_finish_reached are enqueued without waiting; the host
    comes back for the state only at the pruning steps, and notices that the batch has drained through
    sart_active_count_hint (polled every `poll_every` steps; it lags, so a few empty steps may be enqueued).
    graph=True: the three calls are recorded once into a HIP graph that reads the step's K, V and Q from fixed
    buffers (the host copies each step's inputs there, without waiting) and is replayed once per step.
    out: optional float32 device tensor [R*Nb, Hq, d] (rows by handle).  on_step(s, cache, out): hook after each
    step's calls are enqueued (tests; a hook that reads `out` waits for the device itself).
    Returns dict(branch_steps, steps_enqueued)."""
    import torch
    Nb, R = cache.Nb, cache.max_req
    H = R * Nb
    _, n_view = cache.device_views()
    tdev = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).cuda()
    q1 = query(1)
    if out is None:
        out = torch.empty(q1.shape, dtype=torch.float32, device="cuda")
    count = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert cache.sync_status() == 0                     # the hint below is current from here on

    def body(k, v, q):
        cache.append_active_by_handle(k, v)
        cache.decode_attention_by_handle(q, out)
        count.add_(n_view)                              # branches decoded in this step
        cache.finish_reached(tdev)

    drained = [False]

    def maybe_prune(s, event):
        if not (prune_every and s % prune_every == 0):
            return event
        st = cache.get_state(fields=("n_active", "active_handles", "req_counters"))
        n = int(st["n_active"][0])
        drained[0] = n == 0
        if n:
            act_dev = torch.from_numpy(st["active_handles"][:n].astype(np.int64)).cuda()
            cap = np.where(st["req_counters"][:, 0] == 0, Nb // 2, Nb - 1).astype(np.int32)
            cache.prune_branches(DROP_LOWEST_K, scores(event)[act_dev].contiguous(), k=prune_k, max_pruned=cap)
        return event + 1

    event, steps = 0, 0
    g = None
    if graph:
        k1, v1 = step_kv(1)
        src_k, src_v, src_q = torch.empty_like(k1), torch.empty_like(v1), torch.empty_like(q1)

        def load(s):
            k, v = step_kv(s)
            src_k.copy_(k); src_v.copy_(v); src_q.copy_(query(s))
    for s in range(1, n_steps + 1):
        if drained[0] or (s % poll_every == 0 and cache.active_count_hint() == 0):
            break
        if not graph:
            k, v = step_kv(s)
            body(k, v, query(s))
        elif s == 1:
            # step 1 runs eagerly on a side stream (the warm-up a capture needs), step 2 is recorded
            load(1)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                body(src_k, src_v, src_q)
            torch.cuda.current_stream().wait_stream(side)
        else:
            load(s)
            if g is None:
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    body(src_k, src_v, src_q)
            g.replay()
        steps += 1
        if on_step:
            on_step(s, cache, out)
        event = maybe_prune(s, event)
    torch.cuda.synchronize()
    return {"branch_steps": int(count.item()), "steps_enqueued": steps}
