"""Algorithm 1 (the paper's scheduling workflow) on the CPU oracle cache
(TEST INFRASTRUCTURE; shares no code with the HIP library's scheduler).

Written after the paper's pseudo-code: `meta` is the per-request dictionary of
Algorithm 1 (Prefill: phase explore, threshold alpha, max_num_pruned beta,
counters 0); Decode runs up to T steps, then for every involved request
switches the phase when a branch completed (threshold alpha' = reward of the
first completed branch, max_num_pruned N-1), counts completed branches, prunes
incomplete ones whose reward is below the threshold while num_pruned is under
the cap, and answers the request when num_completed >= M or num_completed +
num_pruned == N; the answer is the completed branch with the highest reward
(Section 5.1).  Readings shared with the product:
completion and early stop act at the step they happen, a request's branches are
admitted together when N more fit under B and a window's worth of pages is free,
"first completed" = earliest step then lowest branch index.
"""
from __future__ import annotations

import numpy as np

from . import OK, SEQ_BRANCH, SEQ_PREFIX, THRESHOLD


def serve(cache, *, N, M, alpha, beta, B, T, arrivals, prompt_kv, targets, step_kv, reward, query=None,
          max_rounds=10_000, on_round=None, on_step=None):
    """Returns (answers, stats).  answers[r] = dict(done_round, done_step, answer, answer_reward,
    completed=[(handle, step)...], admitted_round)."""
    pt = cache.pt
    request_queue = list(arrivals)
    meta = {}
    answers = {}
    generated = {}
    step = 0
    stats = dict(branch_steps=0, decode_steps=0, rounds=0, max_active=0, min_free_pages=cache.num_pages)
    pages_per_window = T // pt + 2

    def active_list():
        st = cache.state()
        n = int(st["n_active"][0])
        return st, [int(h) for h in st["active_handles"][:n]]

    for rnd in range(max_rounds):
        st, current_batch = active_list()
        # fill the batch
        while request_queue and request_queue[0][1] <= rnd and len(current_batch) + N <= B:
            i = request_queue[0][0]
            K, V = prompt_kv(i)
            if int(st["free_top"][0]) < -(-len(K) // pt) + (len(current_batch) + N) * pages_per_window:
                break
            request_queue.pop(0)
            assert cache.append(SEQ_PREFIX, [i], [len(K)], K, V) == OK            # Prefill(i)
            meta[i] = dict(phase="explore", threshold=alpha, max_num_pruned=beta, num_completed=0, num_pruned=0,
                           first=None, completed=[], admitted=rnd)
            for j in range(N):
                generated[i * N + j] = 0
            st, current_batch = active_list()
        if not current_batch:
            if not request_queue:
                break
            continue
        stats["max_active"] = max(stats["max_active"], len(current_batch))
        # Decode(current_batch, T)
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
                st, current_batch = active_list()
        # bookkeeping every T steps
        st, current_batch = active_list()
        stats["min_free_pages"] = min(stats["min_free_pages"], int(st["free_top"][0]))
        for i, m in meta.items():
            if m["phase"] == "explore" and m["first"] is not None:
                m.update(phase="exploitation", threshold=float(reward(np.array([m["first"]]), rnd)[0]),
                         max_num_pruned=N - 1)
        if current_batch:
            thr = np.full(cache.max_req, alpha, np.float32)
            cap = np.full(cache.max_req, beta, np.int32)
            for i, m in meta.items():
                thr[i], cap[i] = m["threshold"], m["max_num_pruned"]
            scores = reward(np.array(current_batch), rnd).astype(np.float32)
            assert cache.prune(THRESHOLD, scores, threshold=thr, max_pruned=cap) == OK
            st, current_batch = active_list()
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
                                  completed=list(m["completed"]), admitted_round=m["admitted"])
        stats["rounds"] = rnd + 1
        if on_round:
            on_round(rnd, cache, meta)
        if len(answers) == len(arrivals) and not request_queue:
            break
    return answers, stats
