"""Algorithm 1 of the paper (the SART scheduling workflow) as a host loop over
the HIP library: continuous batching of branches, redundant sampling with early
stopping, and two-phase dynamic pruning.

What follows the paper:
  * Main scheduling workflow: while the current batch holds fewer than B
    branches, an awaiting branch is taken from the branch queue; if there is
    none, the next awaiting request is prefilled, which puts its N branches into
    the branch queue; if there is neither, decoding goes on with a smaller
    batch.  Then the batch decodes for up to T steps.  The batch is filled
    branch by branch, so the branches of a request need not start together
    (Section 4, last paragraph): the library keeps such branches WAITING (they
    hold the prompt, not a row of the batch) until sart_start_branches.
  * Prefill: meta[i] = {explore, threshold alpha, max_num_pruned beta, 0, 0}
    (Algorithm 1, Prefill).
  * After the T steps, per request involved in the batch: if it is still
    exploring and a branch completed, switch to the exploitation phase with
    threshold alpha' = reward of the first completed branch and max_num_pruned
    = N - 1; count completed branches; prune an incomplete branch iff
    num_pruned < max_num_pruned and its reward < threshold; the request is
    answered when num_completed >= M or num_completed + num_pruned == N
    (Algorithm 1, Decode; Section 3, Solution 2).
  * The answer is the completed branch with the highest reward (Section 5.1).
  * KV of a branch is released as soon as it completes, is pruned or is
    early-stopped; the prompt's when the last branch is gone (Section 4).

Readings where the paper leaves room:
  * N and M are called Nb and Q here; both queues are first-in first-out.
  * A branch's completion is seen at the decode step it happens (its KV is
    released at once, and the Q-th completion ends the request's other branches
    at that step, awaiting ones included); rewards, the phase switch, pruning
    and answers come once per T steps, as the paper says.
  * "First completed branch": earliest step, ties to the lowest branch index.
  * Awaiting branches have generated nothing: they are neither scored nor pruned.
  * B is configured for the workload (Section 5.1), so the pool is taken to hold
    B branches; a pool that runs out of pages raises the library's error.
Rewards and completion lengths come from the caller (synthetic stand-ins for
the reward model and the language model).
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field

import numpy as np

from .binding import SEQ_BRANCH, SEQ_PREFIX, THRESHOLD, WAITING


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
    started: dict = field(default_factory=dict)     # handle -> step of its first token
    answer: int = -1                                # handle of the chosen branch, -1 if none completed
    answer_reward: float = float("nan")


class _Batch:
    """Host view of the library's batch: the active handles in active order, refreshed after calls that change it."""

    def __init__(self, cache):
        self.cache = cache
        self.refresh()

    def refresh(self):
        s = self.cache.get_state(fields=("n_active", "active_handles", "free_top", "req_counters", "branch_state"))
        self.n = int(s["n_active"][0])
        self.handles = s["active_handles"][:self.n].copy()
        self.free_pages = int(s["free_top"][0])
        self.completed, self.pruned = s["req_counters"][:, 0].copy(), s["req_counters"][:, 1].copy()
        self.state = s["branch_state"]


def serve(cache, params: SartParams, *, arrivals, prompt_kv, targets, step_kv, query, reward, max_rounds=10_000,
          on_round=None, on_step=None):
    """Runs Algorithm 1 until every request in `arrivals` is answered.

    cache: a SartCache created with start_waiting=True.
    arrivals: list of (request id, round at which it is in the request queue), first come first served.
    prompt_kv(r) -> (K, V) of the prompt; targets[handle] = generated tokens at which the branch completes;
    step_kv(step) / query(step) -> device tensors by handle; reward(handles, round) -> float32 rewards.
    on_round(round, cache, info): hook after each maintenance round; on_step(step, cache, active handles,
    attention output): hook after each decode step (tests).
    Returns (results by request id, stats)."""
    import torch
    Nb, R = cache.Nb, cache.max_req
    assert params.nb == Nb and cache.Q == params.quota
    results = {r: RequestResult(r) for r, _ in arrivals}
    request_queue = deque(arrivals)
    branch_queue = deque()
    exploring = np.ones(R, bool)                    # meta: phase
    threshold = np.full(R, params.alpha, np.float32)
    max_pruned = np.full(R, params.beta, np.int32)
    gen = np.zeros(R * Nb, np.int64)                # tokens generated per branch
    first_done = {}                                 # request -> handle of its first completed branch
    answered = set()
    step = 0
    stats = {"branch_steps": 0, "decode_steps": 0, "rounds": 0, "max_active": 0, "min_free_pages": cache.num_pages}
    batch = _Batch(cache)

    for rnd in range(max_rounds):
        # ---- main workflow: fill the batch from the branch queue, else by prefilling a request ---------------
        while branch_queue and batch.state[branch_queue[0]] != WAITING:
            branch_queue.popleft()                  # its request was answered meanwhile
        room = params.batch - batch.n
        while room > 0:
            if branch_queue:
                b = branch_queue.popleft()
                if batch.state[b] != WAITING:
                    continue
                cache.start_branches([b])           # it takes its place behind its request's rows in the batch
                results[b // Nb].started[b] = step + 1
                room -= 1
            elif request_queue and request_queue[0][1] <= rnd:
                r = request_queue.popleft()[0]
                K, V = prompt_kv(r)
                cache.append_tokens(SEQ_PREFIX, [r], [K.shape[0]], K, V)          # Prefill(r)
                results[r].admitted_round = rnd
                branch_queue.extend(r * Nb + j for j in range(Nb))
                batch.refresh()
            else:
                break
        batch.refresh()
        if batch.n == 0:
            if not request_queue:
                break
            continue                                # nothing to decode yet: wait for the next arrival
        stats["max_active"] = max(stats["max_active"], batch.n)
        # ---- Decode: batch decoding for up to T steps -----------------------------------------------------
        for _ in range(params.window):
            if batch.n == 0:
                break
            step += 1
            act = batch.handles
            act_dev = torch.from_numpy(act.astype(np.int64)).cuda()
            K, V = step_kv(step)
            cache.append_tokens(SEQ_BRANCH, None, None, K[act_dev], V[act_dev])
            out = cache.decode_attention(query(step)[act_dev])
            if on_step:
                on_step(step, cache, act, out)
            gen[act] += 1
            stats["branch_steps"] += batch.n
            stats["decode_steps"] += 1
            fin = act[gen[act] == targets[act]]
            if len(fin):
                for b in fin:                       # active order: ascending branch index within a request
                    results[int(b) // Nb].completed.append((int(b), step))
                    first_done.setdefault(int(b) // Nb, int(b))
                cache.finish_branch(fin)
                batch.refresh()
        # ---- Decode, after the steps: rewards, phase switch, pruning, answers --------------------------------
        batch.refresh()
        stats["min_free_pages"] = min(stats["min_free_pages"], batch.free_pages)
        for r, b in first_done.items():
            if exploring[r]:
                exploring[r] = False
                threshold[r] = reward(np.array([b]), rnd)[0]
                max_pruned[r] = Nb - 1
        if batch.n:
            sc = reward(batch.handles, rnd).astype(np.float32)
            cache.prune_branches(THRESHOLD, sc, threshold=threshold, max_pruned=max_pruned)
            batch.refresh()
        for r, res in results.items():
            if r in answered or res.admitted_round < 0:
                continue
            if batch.completed[r] >= params.quota or batch.completed[r] + batch.pruned[r] == Nb:
                answered.add(r)
                res.done_round, res.done_step = rnd, step
                if res.completed:
                    hs = np.array([h for h, _ in res.completed])
                    rw = reward(hs, rnd)
                    k = int(np.argmax(rw))          # first maximum: earliest completed among equals
                    res.answer, res.answer_reward = int(hs[k]), float(rw[k])
        stats["rounds"] = rnd + 1
        if on_round:
            on_round(rnd, cache, {"active": batch.handles, "threshold": threshold.copy(), "max_pruned": max_pruned.copy()})
        if len(answered) == len(results) and not request_queue:
            break
    return results, stats
