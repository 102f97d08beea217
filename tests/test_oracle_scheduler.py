"""Pins of the oracle-side Algorithm 1 driver against what the paper fixes."""
import numpy as np

import oracle as orc
from helpers import check_invariants, make_oracle
from oracle.scheduler import serve


def _run(*, R=10, N=8, M=4, alpha=0.5, beta=4, B=32, T=10, seed=0, arrive_every=1, reward_fn=None, targets=None,
         pt=4, P=5, on_step=None):
    rng = np.random.default_rng(seed)
    targets = rng.integers(3, 60, size=R * N) if targets is None else targets
    num_pages = B * (int(targets.max()) // pt + T // pt + 4) + R * 2 + 16
    o = make_oracle(Hq=1, Hkv=1, d=8, pt=pt, num_pages=num_pages, max_req=R, Nb=N, Q=M,
                    max_bp=int(targets.max()) // pt + 2, max_pp=2, start_waiting=True)
    one = np.ones((R * N, 1, 8), np.float32)
    table = np.random.default_rng(seed + 1).random((400, R * N)).astype(np.float32)
    reward = reward_fn or (lambda hs, rnd: table[rnd % 400, hs])
    log = []

    def on_round(rnd, cache, meta):
        st = cache.state()
        check_invariants(st, pt=pt, num_pages=num_pages, Nb=N, max_req=R)
        assert st["n_active"][0] <= B
        for i, m in meta.items():
            # Algorithm 1: at most beta pruned while exploring, at most N-1 ever
            assert m["num_pruned"] <= (beta if m["phase"] == "explore" else N - 1)
        log.append({i: dict(m) for i, m in meta.items()})

    answers, stats = serve(o, N=N, M=M, alpha=alpha, beta=beta, B=B, T=T,
                           arrivals=[(r, r * arrive_every) for r in range(R)],
                           prompt_kv=lambda r: (one[:P], one[:P]), targets=targets,
                           step_kv=lambda s: (one, one), reward=reward, on_round=on_round, on_step=on_step)
    return o, answers, stats, log, targets, reward, num_pages


def test_every_request_is_answered_and_memory_returns():
    o, answers, stats, log, targets, reward, num_pages = _run()
    assert sorted(answers) == list(range(10))
    st = o.state()
    assert st["n_active"][0] == 0 and st["free_top"][0] == num_pages
    for r, a in answers.items():
        c, p = st["req_counters"][r]
        assert c >= 4 or c + p == 8                       # Algorithm 1's output condition
        assert len(a["completed"]) == c
        if a["completed"]:                                 # answer = completed branch with the highest reward
            hs = np.array([h for h, _ in a["completed"]])
            assert a["answer"] == hs[np.argmax(reward(hs, a["done_round"]))]
        else:
            assert a["answer"] == -1
    assert stats["max_active"] <= 32


def test_without_pruning_a_request_needs_the_Mth_shortest_branch():
    """Equal rewards never prune (the predicate is a strict <, in both phases); every request admitted at once:
    the step at which a request's M-th branch completes is the M-th smallest length (Section 3, Solution 1 /
    Lemma 1)."""
    R, N, M, T = 4, 8, 4, 7
    o, answers, stats, log, targets, _, _ = _run(R=R, N=N, M=M, alpha=0.5, B=R * N, T=T, arrive_every=0,
                                                 reward_fn=lambda hs, rnd: np.full(len(hs), 0.7, np.float32))
    for r in range(R):
        kth = int(np.sort(targets[r * N:(r + 1) * N])[M - 1])
        done = [s for _, s in answers[r]["completed"]]
        assert max(done) == kth and len(done) >= M
        assert answers[r]["done_round"] == (kth - 1) // T       # answered at the end of that window
    assert o.state()["req_counters"][:, 1].sum() == 0


def test_two_phase_threshold_follows_the_first_completed_branch():
    """Rewards fixed per branch: before the first completion the threshold is alpha and at most beta branches go;
    afterwards it is the first completed branch's reward and up to N-1 may go."""
    N = 8
    base = np.array([0.9, 0.45, 0.6, 0.3, 0.7, 0.2, 0.8, 0.65], np.float32)
    targets = np.array([12, 50, 50, 50, 50, 50, 50, 50])
    o, answers, stats, log, *_ = _run(R=1, N=N, M=4, alpha=0.5, beta=2, B=8, T=5, targets=targets,
                                      reward_fn=lambda hs, rnd: base[np.asarray(hs) % N])
    # round 0 (explore): rewards < 0.5 are branches 1, 3, 5 in active order; the cap beta = 2 stops after 1 and 3
    assert log[0][0]["phase"] == "explore" and log[0][0]["num_pruned"] == 2
    st_states = o.state()["branch_state"]
    assert st_states[1] == orc.PRUNED and st_states[3] == orc.PRUNED
    # branch 0 completes at step 12 (window 2): threshold becomes 0.9, cap N-1: every other live branch is pruned
    assert log[2][0]["phase"] == "exploitation" and abs(log[2][0]["threshold"] - 0.9) < 1e-6
    assert log[2][0]["max_num_pruned"] == N - 1 and log[2][0]["num_pruned"] == N - 1
    assert answers[0]["answer"] == 0 and answers[0]["done_round"] == 2


def test_fcfs_admission_under_batch_limit():
    """B = 16 holds two requests of N = 8: the third is prefilled only after one left."""
    o, answers, stats, log, *_ = _run(R=5, N=8, M=4, B=16, T=6, arrive_every=0, seed=3)
    adm = [answers[r]["admitted_round"] for r in range(5)]
    assert adm[0] == 0 and adm[1] == 0 and adm[2] > 0
    assert adm == sorted(adm)                                   # first come, first served
    assert stats["max_active"] <= 16


def test_branches_of_a_request_need_not_start_together():
    """B = 3 with N = 2: the batch is filled branch by branch (Algorithm 1, main workflow), so request 1 gets
    one branch into the first batch and the other waits in branch_queue until a place is free.  Worked by hand
    (no pruning: equal rewards; M = N = 2; T = 4; tokens to generate b00 6, b01 3, b10 5, b11 2):
      round 0: Prefill(0) queues b00 b01, both start; Prefill(1) queues b10 b11, b10 starts, the batch is full;
               steps 1-4: b01 completes at step 3.
      round 1: b11 starts (its first token is step 5); b10 completes at step 5; b00 and b11 complete at step 6.
    So request 1's earliest completed branch (b10, 5 tokens, step 5) is not its shortest (b11, 2 tokens, step 6):
    Section 4, last paragraph."""
    batches = {}
    o, answers, stats, log, *_ = _run(R=2, N=2, M=2, B=3, T=4, arrive_every=0, targets=np.array([6, 3, 5, 2]),
                                      reward_fn=lambda hs, rnd: np.full(len(hs), 0.7, np.float32),
                                      on_step=lambda s, c, batch: batches.__setitem__(s, list(batch)))
    assert batches[1] == [0, 1, 2] and batches[4] == [0, 2]          # b01 left after step 3
    assert batches[5] == [0, 2, 3] and batches[6] == [0, 3]          # b11 joined behind its request's b10
    assert answers[0]["completed"] == [(1, 3), (0, 6)] and answers[1]["completed"] == [(2, 5), (3, 6)]
    assert answers[0]["started"] == {0: 1, 1: 1} and answers[1]["started"] == {2: 1, 3: 5}
    assert answers[0]["done_round"] == 1 and answers[1]["done_round"] == 1 and answers[1]["done_step"] == 6
    assert stats["max_active"] == 3 and stats["branch_steps"] == 3 + 3 + 3 + 2 + 3 + 2


def test_early_stop_ends_the_awaiting_branches_too():
    """N = 3, M = 1, B = 2: b02 is still in branch_queue when b01 completes at step 2; the request is answered and
    b00 (running) and b02 (never started) are both ended, the prompt is released, and request 1 takes the places."""
    o, answers, stats, log, *_ = _run(R=2, N=3, M=1, B=2, T=3, arrive_every=0, targets=np.array([9, 2, 4, 5, 5, 1]),
                                      reward_fn=lambda hs, rnd: np.full(len(hs), 0.7, np.float32))
    st = o.state()
    assert list(st["branch_state"][:3]) == [orc.EARLY_STOPPED, orc.COMPLETED, orc.EARLY_STOPPED]
    assert answers[0]["completed"] == [(1, 2)] and answers[0]["started"] == {0: 1, 1: 1} and answers[0]["answer"] == 1
    # round 0 decodes 2 steps only (the batch is empty after step 2); request 1 is prefilled in round 1 (the batch
    # was full in round 0): b10, b11 start at step 3 and both complete at step 7 (5 tokens each); the first of
    # them ends the request: b12 never starts
    assert answers[1]["admitted_round"] == 1 and answers[1]["started"] == {3: 3, 4: 3}
    assert answers[1]["completed"][0][1] == 7 and st["branch_state"][5] == orc.EARLY_STOPPED
    assert st["n_active"][0] == 0 and np.all(st["prefix_refcnt"] == 0)
