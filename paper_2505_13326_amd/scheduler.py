"""Algorithm 1 of the paper (the SART scheduling workflow) as a host loop over
the HIP library: continuous batching of branches, redundant sampling with early
stopping, and two-phase dynamic pruning.

What follows the paper:
  * Main workflow: while the batch has room, admit work (awaiting branches
    first, else prefill the next awaiting request, which adds its N branches),
    then decode for up to T steps (Algorithm 1, main loop and Decode).
  * Prefill: meta[i] = {explore, threshold alpha, max_num_pruned beta, 0, 0}
    (Algorithm 1, Prefill).
  * Every T steps, per involved request: if it is still exploring and a branch
    completed, switch to the exploitation phase with threshold alpha' = reward
    of the first completed branch and max_num_pruned = N - 1; count completed
    branches; prune an incomplete branch iff num_pruned < max_num_pruned and its
    reward < threshold; the request is answered when num_completed >= M or
    num_completed + num_pruned == N (Algorithm 1, Decode; Section 3, Solution 2).
  * The answer is the completed branch with the highest reward (Section 5.1).
  * KV of a branch is released as soon as it completes, is pruned or is
    early-stopped; the prompt's when the last branch is gone (Section 4).

Readings where the paper leaves room:
  * N and M are called Nb and Q here.
  * A branch's completion is seen at the decode step it happens (its KV is
    released at once, and the Q-th completion early-stops the request's other
    branches at that step); rewards, the phase switch and pruning run every T
    steps, as the paper says.
  * A request's Nb branches enter the batch together: a request is prefilled when
    Nb more branches fit under B and the pool holds enough free pages for one
    more window; so there is no separate queue of awaiting branches.
  * "First completed branch": earliest step, ties to the lowest branch index.
Rewards and completion lengths come from the caller (synthetic stand-ins for
the reward model and the language model).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from .binding import SEQ_BRANCH, SEQ_PREFIX, THRESHOLD


@dataclass
class SartParams:
    nb: int                 # branches sampled per request (paper's N)
    quota: int              # completions that end a request (paper's M), default N/2
    alpha: float = 0.5      # first-phase pruning threshold
    beta: int = -1          # first-phase cap on pruned branches, default N/2
    batch: int = 64         # B: branches decoded together at most
    window: int = 400       # T: decode steps between maintenance rounds

    def __post_init__(self):
        if self.beta < 0:
            self.beta = self.nb // 2


@dataclass
class RequestResult:
    request: int
    admitted_round: int = -1
    done_round: int = -1
    done_step: int = -1
    completed: list = field(default_factory=list)   # (handle, step) in completion order
    answer: int = -1                                # handle of the chosen branch, -1 if none completed
    answer_reward: float = float("nan")


def serve(cache, params: SartParams, *, arrivals, prompt_kv, targets, step_kv, query, reward, max_rounds=10_000,
          on_round=None, on_step=None):
    """Runs Algorithm 1 until every request in `arrivals` is answered.

    arrivals: list of (request id, round at which it is in the request queue), FCFS in list order.
    prompt_kv(r) -> (K, V) of the prompt; targets[handle] = generated tokens at which the branch completes;
    step_kv(step) / query(step) -> device tensors by handle; reward(handles, round) -> float32 rewards.
    on_round(round, cache, info): hook after each maintenance round; on_step(step, cache, active handles,
    attention output): hook after each decode step (tests).
    Returns (results by request id, stats)."""
    import torch
    Nb, R = cache.Nb, cache.max_req
    assert params.nb == Nb and cache.Q == params.quota
    pt = cache.pt
    results = {r: RequestResult(r) for r, _ in arrivals}
    queue = list(arrivals)
    phase_explore = np.ones(R, bool)
    threshold = np.full(R, params.alpha, np.float32)
    max_pruned = np.full(R, params.beta, np.int32)
    gen = np.zeros(R * Nb, np.int64)                # tokens generated per branch
    first_done = {}                                 # request -> (step, handle) of its first completion
    answered = set()
    step = 0
    stats = {"branch_steps": 0, "decode_steps": 0, "rounds": 0, "max_active": 0, "min_free_pages": cache.num_pages}
    window_pages = params.window // pt + 2          # pages a branch can need within one window

    def state():
        s = cache.get_state(fields=("n_active", "active_handles", "free_top", "req_counters"))
        n = int(s["n_active"][0])
        return s, n, s["active_handles"][:n].copy()

    for rnd in range(max_rounds):
        s, nA, act = state()
        # ---- fill the batch: prefill awaiting requests while their branches fit -------------------
        while queue and queue[0][1] <= rnd and nA + Nb <= params.batch:
            r = queue[0][0]
            K, V = prompt_kv(r)
            need = -(-K.shape[0] // pt) + (nA + Nb) * window_pages
            if int(s["free_top"][0]) < need:
                break                               # memory bound: wait for branches to leave
            queue.pop(0)
            cache.append_tokens(SEQ_PREFIX, [r], [K.shape[0]], K, V)
            results[r].admitted_round = rnd
            s, nA, act = state()
        if nA == 0:
            if not queue:
                break
            continue                                # nothing to decode yet: wait for the next arrival
        stats["max_active"] = max(stats["max_active"], nA)
        # ---- decode for up to T steps -------------------------------------------------------------
        for _ in range(params.window):
            if nA == 0:
                break
            step += 1
            act_dev = torch.from_numpy(act.astype(np.int64)).cuda()
            K, V = step_kv(step)
            cache.append_tokens(SEQ_BRANCH, None, None, K[act_dev], V[act_dev])
            out = cache.decode_attention(query(step)[act_dev])
            if on_step:
                on_step(step, cache, act, out)
            gen[act] += 1
            stats["branch_steps"] += nA
            stats["decode_steps"] += 1
            fin = act[gen[act] == targets[act]]
            if len(fin):
                for b in fin:                       # ascending active order = ascending branch index per request
                    r = int(b) // Nb
                    results[r].completed.append((int(b), step))
                    first_done.setdefault(r, (step, int(b)))
                cache.finish_branch(fin)
                s, nA, act = state()
        # ---- maintenance round: rewards, phase switch, pruning, answers ---------------------------
        s, nA, act = state()
        stats["min_free_pages"] = min(stats["min_free_pages"], int(s["free_top"][0]))
        for r, (_, b) in first_done.items():
            if phase_explore[r]:
                phase_explore[r] = False
                threshold[r] = reward(np.array([b]), rnd)[0]
                max_pruned[r] = Nb - 1
        if nA:
            sc = reward(act, rnd).astype(np.float32)
            cache.prune_branches(THRESHOLD, sc, threshold=threshold, max_pruned=max_pruned)
            s, nA, act = state()
        c, p = s["req_counters"][:, 0], s["req_counters"][:, 1]
        for r, res in results.items():
            if r in answered or res.admitted_round < 0:
                continue
            if c[r] >= params.quota or c[r] + p[r] == Nb:
                answered.add(r)
                res.done_round, res.done_step = rnd, step
                if res.completed:
                    hs = np.array([h for h, _ in res.completed])
                    rw = reward(hs, rnd)
                    k = int(np.argmax(rw))          # first maximum: earliest completed among equals
                    res.answer, res.answer_reward = int(hs[k]), float(rw[k])
        stats["rounds"] = rnd + 1
        if on_round:
            on_round(rnd, cache, {"active": act, "threshold": threshold.copy(), "max_pruned": max_pruned.copy()})
        if len(answered) == len(results) and not queue:
            break
    return results, stats
