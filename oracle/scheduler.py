"""Algorithm 1 (the paper's scheduling workflow) on the CPU oracle cache
(TEST INFRASTRUCTURE; shares no code with the HIP library's scheduler).

Written after the pseudo-code, in its order and with its names:

  main workflow   while the current batch holds fewer than B branches: pop an
                  awaiting branch from branch_queue into it; if there is none,
                  Prefill the next awaiting request (which pushes its N branches
                  into branch_queue); if there is neither, go on with a smaller
                  batch.  Then Decode(current_batch, T).
  Prefill(i)      prefill request i; meta[i] = {phase explore, threshold alpha,
                  max_num_pruned beta, num_completed 0, num_pruned 0}; push
                  b_i1 .. b_iN into branch_queue.
  Decode          batch decoding for up to T steps; then, for every request
                  involved in the batch: if it is exploring and a branch of it
                  completed, switch to the exploitation phase (threshold alpha' =
                  reward of the first completed branch, max_num_pruned N - 1);
                  count and remove its completed branches; prune an incomplete
                  branch iff num_pruned < max_num_pruned and its reward <
                  threshold; output the request when num_completed >= M or
                  num_completed + num_pruned == N.
  answer          the completed branch with the highest reward (Section 5.1).

Because the batch is filled branch by branch, a request's branches need not
start together (Section 4, last paragraph): with B not a multiple of N a request
sits half in the batch and half in branch_queue.

Readings where the pseudo-code leaves room (the same as the product's, stated
there too): both queues are first-in first-out; a branch that completes leaves
the batch at the step it completes, its KV is released at once, and the M-th
completion ends the request's other branches at that step, awaiting ones
included (Section 3, Solution 1; Section 4: immediate release) while rewards,
the phase switch, pruning and outputs happen once per Decode, after its T steps;
"first completed" = earliest step, ties to the lowest branch index; awaiting
branches have generated nothing, so they are neither scored nor pruned.
"""
from __future__ import annotations

import numpy as np

from . import OK, SEQ_BRANCH, SEQ_PREFIX, THRESHOLD, WAITING


def serve(cache, *, N, M, alpha, beta, B, T, arrivals, prompt_kv, targets, step_kv, reward, query=None,
          max_rounds=10_000, on_round=None, on_step=None):
    """cache: an OracleCache created with start_waiting=True.  arrivals: [(request, round at which it is in the
    request queue)], first come first served.  Returns (answers, stats); answers[i] = dict(done_round, done_step,
    answer, answer_reward, completed=[(handle, step)...], admitted_round, started={handle: step of its first token})."""
    request_queue = list(arrivals)
    branch_queue = []
    meta = {}
    answers = {}
    generated = {}
    step = 0
    stats = dict(branch_steps=0, decode_steps=0, rounds=0, max_active=0, min_free_pages=cache.num_pages)

    def batch_now():
        st = cache.state()
        n = int(st["n_active"][0])
        return st, [int(h) for h in st["active_handles"][:n]]

    def prefill(i, rnd):
        K, V = prompt_kv(i)
        assert cache.append(SEQ_PREFIX, [i], [len(K)], K, V) == OK
        meta[i] = dict(phase="explore", threshold=alpha, max_num_pruned=beta, num_completed=0, num_pruned=0,
                       first=None, completed=[], admitted=rnd, started={})
        for j in range(N):
            branch_queue.append(i * N + j)
            generated[i * N + j] = 0

    for rnd in range(max_rounds):
        # ---- main workflow: fill the batch ------------------------------------------------------------------
        st, current_batch = batch_now()
        # awaiting branches of requests that were ended meanwhile are no longer awaiting
        branch_queue = [b for b in branch_queue if st["branch_state"][b] == WAITING]
        while len(current_batch) < B:
            if branch_queue:
                b = branch_queue.pop(0)
                assert cache.start([b]) == OK
                current_batch.append(b)
                meta[b // N]["started"][b] = step + 1
            elif request_queue and request_queue[0][1] <= rnd:
                prefill(request_queue.pop(0)[0], rnd)
            else:
                break
        st, current_batch = batch_now()
        if not current_batch:
            if not request_queue:
                break
            continue                                    # nothing to decode yet: wait for the next arrival
        stats["max_active"] = max(stats["max_active"], len(current_batch))
        involved = sorted({b // N for b in current_batch})
        # ---- Decode: batch decoding for up to T steps -------------------------------------------------------
        for _ in range(T):
            if not current_batch:
                break
            step += 1
            K, V = step_kv(step)
            assert cache.append(SEQ_BRANCH, None, None, K[current_batch], V[current_batch]) == OK
            if on_step:
                on_step(step, cache, current_batch)
            stats["branch_steps"] += len(current_batch)
            stats["decode_steps"] += 1
            done_now = []
            for b in current_batch:
                generated[b] += 1
                if generated[b] == targets[b]:
                    done_now.append(b)
            if done_now:
                for b in done_now:
                    m = meta[b // N]
                    m["completed"].append((b, step))
                    if m["first"] is None:
                        m["first"] = b
                assert cache.finish(done_now) == OK
                st, current_batch = batch_now()
        # ---- Decode: per involved request, after the T steps -------------------------------------------------
        st, current_batch = batch_now()
        stats["min_free_pages"] = min(stats["min_free_pages"], int(st["free_top"][0]))
        for i in involved:
            m = meta[i]
            if m["phase"] == "explore" and m["first"] is not None:
                m.update(phase="exploitation", threshold=float(reward(np.array([m["first"]]), rnd)[0]), max_num_pruned=N - 1)
        if current_batch:
            thr = np.full(cache.max_req, alpha, np.float32)
            cap = np.full(cache.max_req, beta, np.int32)
            for i, m in meta.items():
                thr[i], cap[i] = m["threshold"], m["max_num_pruned"]
            scores = reward(np.array(current_batch), rnd).astype(np.float32)
            assert cache.prune(THRESHOLD, scores, threshold=thr, max_pruned=cap) == OK
            st, current_batch = batch_now()
        for i, m in meta.items():
            m["num_completed"], m["num_pruned"] = int(st["req_counters"][i, 0]), int(st["req_counters"][i, 1])
            if i in answers:
                continue
            if m["num_completed"] >= M or m["num_completed"] + m["num_pruned"] == N:
                best, best_reward = -1, float("nan")
                if m["completed"]:
                    hs = np.array([h for h, _ in m["completed"]])
                    rw = reward(hs, rnd)
                    k = int(np.argmax(rw))
                    best, best_reward = int(hs[k]), float(rw[k])
                answers[i] = dict(done_round=rnd, done_step=step, answer=best, answer_reward=best_reward,
                                  completed=list(m["completed"]), admitted_round=m["admitted"], started=dict(m["started"]))
        stats["rounds"] = rnd + 1
        if on_round:
            on_round(rnd, cache, meta)
        if len(answers) == len(arrivals) and not request_queue:
            break
    return answers, stats
