"""A decode step recorded once into a HIP graph and replayed while the batch
changes under it (the step loop of Algorithm 1, Decode, without a host
round-trip per call): append one token to every active branch, attend, and
complete the branches that reached their target length (with the early stop
that follows).  The plan of the step lives on the device, the all-active append
bakes no count into the launch and the completion takes its targets from device
memory, so the same graph serves while branches finish inside it and are pruned
(eagerly) between replays.  Every replay is checked against the oracle."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import GpuEngine, TOL, dims, populate
from helpers import assert_state_equal

pytestmark = pytest.mark.gpu


def test_decode_step_graph_replays_across_finish_and_prune():
    import torch
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=4, nb=8, quota=4, prompt_len=100, length_params=(150, 0.8), length_cap=900)
    L = wl.lengths(cfg)
    steps = 24
    pages = wl.pages_needed(cfg, L, growth_tokens=steps) + 8
    kw = dims(cfg, pages, int(-(-(L.max() + steps) // 16)) + 1)
    fo = wl.free_order(cfg, pages)
    o = orc.OracleCache(free_order=fo, **kw)
    g = GpuEngine(free_order=fo, **kw)
    populate(cfg, [o, g], L)
    H = cfg.n_handles
    # target lengths: a few branches complete on most steps; request 2 reaches its quota of 4 (early stop)
    rng = np.random.default_rng(3)
    targets = (L.reshape(-1) + rng.integers(3, 40, size=H)).astype(np.int32)
    targets[16:20] = L.reshape(-1)[16:20] + np.array([5, 5, 9, 12])
    tdev = torch.from_numpy(targets).cuda()
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()
    kbuf = torch.zeros((H, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    vbuf = torch.zeros_like(kbuf)
    qbuf = torch.zeros((H, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((H, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")

    def active():
        st = o.state()
        return st["active_handles"][:int(st["n_active"][0])]

    def load_inputs(s, act):
        k, v = wl.step_kv(cfg, s)
        n = len(act)
        kbuf[:n].copy_(dev(k[act])); vbuf[:n].copy_(dev(v[act])); qbuf[:n].copy_(dev(wl.query(cfg, s)[act]))
        return k[act], v[act], wl.query(cfg, s)[act]

    n_finished = [0]

    def check(s, act, k, v, q):
        assert o.append(orc.SEQ_BRANCH, None, None, k, v) == orc.OK
        ref = o.attention(q)
        # the oracle completes the same branches from a host list: those whose length reached the target
        st = o.state()
        lens = st["seq_lens"][:len(act)]
        fin = [int(b) for b, n in zip(act, lens) if n >= targets[b]]
        if fin:
            assert o.finish(fin) == orc.OK
            n_finished[0] += len(fin)
        assert g.c.sync_status() == 0
        assert_state_equal(o.state(), g.state())
        got = out[:len(act)].cpu().numpy().astype(np.float64)
        err = float(np.abs(got - ref).max())
        assert np.all(np.isfinite(got)) and err <= TOL["bf16"], f"step {s}: max abs err {err}"

    # step 1 eagerly on a side stream (also the warm-up the capture needs), then record step 2
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    act = active()
    k, v, q = load_inputs(1, act)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        g.c.append_tokens(orc.SEQ_BRANCH, None, None, kbuf, vbuf, all_active=True)
        g.c.decode_attention(qbuf, out=out)
        g.c.finish_reached(tdev)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    check(1, act, k, v, q)

    graph = torch.cuda.CUDAGraph()
    k, v, q = load_inputs(2, act)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        g.c.append_tokens(orc.SEQ_BRANCH, None, None, kbuf, vbuf, all_active=True)
        g.c.decode_attention(qbuf, out=out)
        g.c.finish_reached(tdev)
    graph.replay()                      # capture records, replay runs: this is step 2
    torch.cuda.synchronize()
    check(2, act, k, v, q)

    for s in range(3, steps + 1):
        if s == 8:                      # eager maintenance between replays: the batch shrinks
            fin = [int(act[1]), int(act[-1])]
            assert o.finish(fin) == orc.OK and g.finish(fin) == orc.OK
        if s == 14:
            sc = wl.scores(cfg, 0)[act]
            assert o.prune(orc.DROP_LOWEST_K, sc, k=2) == orc.OK and g.prune(orc.DROP_LOWEST_K, sc, k=2) == orc.OK
        act = active()
        k, v, q = load_inputs(s, act)
        out.fill_(7.0)                  # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        check(s, act, k, v, q)
    assert len(act) < H and n_finished[0] >= 8      # the batch did change under the graph, and inside it
    assert o.state()["req_counters"][:, 0].max() >= cfg.quota       # a request reached its quota: early stop ran

    # the row capacity of an all-active append is checked on the device
    small = kbuf[: len(act) - 1]
    g.c.append_tokens(orc.SEQ_BRANCH, None, None, small, vbuf[: len(act) - 1], all_active=True)
    assert g.c.sync_status() == orc.E_INVALID
    assert_state_equal(o.state(), g.state())


def test_finish_reached_edges():
    """No branch at its target: nothing changes (and an append to another layer may still follow);
    every branch at its target: the cache drains completely."""
    import torch
    cfg = wl.scaled(wl.CONFIGS[2], n_requests=2, nb=4, quota=0, prompt_len=40, length_params=(60, 0.5), length_cap=300)
    L = wl.lengths(cfg)
    pages = wl.pages_needed(cfg, L, growth_tokens=4) + 4
    kw = dims(cfg, pages, int(-(-(L.max() + 4) // 16)) + 1)
    o = orc.OracleCache(**kw)
    g = GpuEngine(n_layers=2, **kw)
    for r in range(cfg.n_requests):
        k, v = wl.prefix_kv(cfg, r)
        assert o.append(orc.SEQ_PREFIX, [r], [cfg.prompt_len], k, v) == orc.OK
        ids = [r * cfg.nb + j for j in range(cfg.nb)]
        ns = [int(L[r, j]) for j in range(cfg.nb)]
        kb, vb = (np.concatenate(x) for x in zip(*[wl.branch_kv(cfg, b, n) for b, n in zip(ids, ns)]))
        assert o.append(orc.SEQ_BRANCH, ids, ns, kb, vb) == orc.OK
        for l in range(2):
            g.c.append_tokens(orc.SEQ_PREFIX, [r], [cfg.prompt_len], k, v, layer=l)
        for l in range(2):
            g.c.append_tokens(orc.SEQ_BRANCH, ids, ns, kb, vb, layer=l)
    assert g.c.sync_status() == 0
    assert_state_equal(o.state(), g.state())
    H = cfg.n_handles
    act = o.state()["active_handles"][:H]
    k, v = wl.step_kv(cfg, 1)
    far = torch.full((H,), 1 << 30, dtype=torch.int32, device="cuda")
    # layer 0 append, a completion call that finds nothing, then the other layer's append: still written
    assert o.append(orc.SEQ_BRANCH, None, None, k[act], v[act]) == orc.OK
    g.c.append_tokens(orc.SEQ_BRANCH, None, None, k[act], v[act], layer=0)
    g.c.finish_reached(far)
    g.c.append_tokens(orc.SEQ_BRANCH, None, None, k[act], v[act], layer=1)
    assert g.c.sync_status() == 0
    assert_state_equal(o.state(), g.state())
    q = wl.query(cfg, 1)[act]
    ref = o.attention(q)
    for l in range(2):
        got = g.c.decode_attention(q, layer=l).cpu().numpy().astype(np.float64)
        assert float(np.abs(got - ref).max()) <= TOL["bf16"]
    # every branch has reached a target of zero tokens: all complete, every page returns
    g.c.finish_reached(torch.zeros(H, dtype=torch.int32, device="cuda"))
    assert o.finish([int(b) for b in act]) == orc.OK
    assert g.c.sync_status() == 0
    st = g.state()
    assert_state_equal(o.state(), st)
    assert int(st["n_active"][0]) == 0 and int(st["free_top"][0]) == pages
