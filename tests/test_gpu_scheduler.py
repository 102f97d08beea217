"""Algorithm 1 end to end: the HIP-side scheduler against the oracle-side one on the same seeded
request stream (continuous batching branch by branch through the branch queue, with B not a multiple of N so that
requests sit half in the batch and half in the queue; early stop; two-phase pruning; pages reused).
Integer state is compared after every maintenance round (digest), attention on sampled rows every step."""
import hashlib

import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import TOL, GpuEngine, dims
from helpers import check_invariants
from oracle.scheduler import serve as oracle_serve

pytestmark = pytest.mark.gpu

KEYS = ("n_active", "active_handles", "seq_lens", "block_tables", "free_stack", "free_top", "prefix_tables",
        "prefix_lens", "prefix_refcnt", "branch_state", "req_counters")


def _digest(st):
    h = hashlib.sha1()
    for k in KEYS:
        h.update(np.ascontiguousarray(st[k]).tobytes())
    return h.hexdigest()


def test_sart_scheduler_matches_oracle():
    import torch
    from paper_2505_13326_amd.scheduler import SartParams, serve
    R, N, M, B, T = 14, 8, 4, 29, 25
    cfg = wl.scaled(wl.CONFIGS[3], n_requests=R, prompt_len=200, quota=M)
    rng = np.random.default_rng(77)
    targets = np.maximum(3, np.rint(60 * np.exp(0.8 * rng.standard_normal(R * N)))).astype(np.int64)
    targets = np.minimum(targets, 400)
    # B is configured for the pool (Section 5.1): room for B branches of the longest length and the live prompts
    max_bp = 400 // 16 + 2
    num_pages = B * max_bp + R * 13
    kw = dims(cfg, num_pages, max_bp, max_pp=13)
    fo = wl.free_order(cfg, num_pages)
    o, g = orc.OracleCache(free_order=fo, start_waiting=True, **kw), GpuEngine(free_order=fo, start_waiting=True, **kw)
    arrivals = [(r, r // 3) for r in range(R)]
    reward_table = np.random.default_rng(5).random((64, R * N)).astype(np.float32)
    reward = lambda hs, rnd: reward_table[rnd % 64, np.asarray(hs)]

    ref_rounds, ref_attn = [], {}

    def o_round(rnd, cache, meta):
        ref_rounds.append(_digest(cache.state()))

    def o_step(step, cache, batch):
        rows = sorted(set([0, len(batch) // 2, len(batch) - 1]))
        ref_attn[step] = (rows, cache.attention(wl.query(cfg, step)[batch], rows=rows))

    ans_o, stats_o = oracle_serve(o, N=N, M=M, alpha=0.5, beta=N // 2, B=B, T=T, arrivals=arrivals,
                                  prompt_kv=lambda r: wl.prefix_kv(cfg, r), targets=targets,
                                  step_kv=lambda s: wl.step_kv(cfg, s), reward=reward, on_round=o_round, on_step=o_step)

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()

    pos, worst = [0], [0.0]

    def g_round(rnd, cache, info):
        st, rc = cache.get_state(with_status=True)
        assert rc == 0
        assert _digest(st) == ref_rounds[pos[0]], f"state differs after round {rnd}"
        check_invariants(st, pt=16, num_pages=num_pages, Nb=N, max_req=R)
        assert st["n_active"][0] <= B
        pos[0] += 1

    def g_step(step, cache, act, out):
        rows, ref = ref_attn[step]
        got = out[torch.as_tensor(rows, device="cuda")].cpu().numpy().astype(np.float64)
        worst[0] = max(worst[0], float(np.abs(got - ref).max()))

    res_g, stats_g = serve(g.c, SartParams(nb=N, quota=M, alpha=0.5, batch=B, window=T), arrivals=arrivals,
                           prompt_kv=lambda r: wl.prefix_kv(cfg, r), targets=targets,
                           step_kv=lambda s: tuple(dev(x) for x in wl.step_kv(cfg, s)),
                           query=lambda s: dev(wl.query(cfg, s)), reward=reward, on_round=g_round, on_step=g_step)
    assert pos[0] == len(ref_rounds)
    assert stats_g == stats_o, (stats_g, stats_o)
    for r in range(R):
        a, b = ans_o[r], res_g[r]
        assert (a["done_round"], a["done_step"], a["answer"], a["admitted_round"]) == \
               (b.done_round, b.done_step, b.answer, b.admitted_round)
        assert a["completed"] == b.completed and a["started"] == b.started
    assert worst[0] <= TOL["bf16"]
    st = g.state()
    assert st["n_active"][0] == 0 and st["free_top"][0] == num_pages
    late = [res_g[r].admitted_round for r in range(R)]
    assert max(l - r // 3 for r, l in enumerate(late)) > 0      # somebody had to queue for room
    split = [r for r in range(R) if len(set(res_g[r].started.values())) > 1]
    assert split, "no request had its branches start at different steps"
    assert stats_g["min_free_pages"] < num_pages - 100           # the pool was in use ...
    assert not np.array_equal(st["free_stack"], fo[::-1])        # ... and its pages came back in another order
    print(f"scheduler: {stats_g}, max abs attention err {worst[0]:.3g}, admitted rounds {late}")
