"""Config 3: the early-stop / prune trace on the GPU against the oracle's own
step loop.  Integer state is compared after EVERY library call (bit-exact, via
a digest of all state arrays); attention is compared on sampled rows at every
step."""
import hashlib

import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import TOL, GpuEngine, compare_attention, dims, populate
from helpers import check_invariants
from oracle.trace import run_trace as oracle_trace

pytestmark = pytest.mark.gpu

KEYS = ("n_active", "active_handles", "seq_lens", "block_tables", "free_stack", "free_top", "prefix_tables",
        "prefix_lens", "prefix_refcnt", "branch_state", "req_counters")


def _digest(st):
    h = hashlib.sha1()
    for k in KEYS:
        h.update(np.ascontiguousarray(st[k]).tobytes())
    return h.hexdigest()


def _sample_rows(nA):
    return sorted(set(list(range(min(4, nA))) + list(range(max(0, nA - 4), nA))))


@pytest.mark.parametrize("size", ["small", "cfg3"])
def test_trace_matches_oracle_after_every_call(size):
    import torch
    from paper_2505_13326_amd.trace import run_trace as gpu_trace
    cfg = wl.CONFIGS[3]
    if size == "small":
        cfg = wl.scaled(cfg, n_requests=5, length_params=(150, 0.8), length_cap=1200, n_steps=130, prune_every=20)
    L = wl.lengths(cfg)
    targets = (L + wl.remaining_tokens(cfg)).reshape(-1)
    num_pages = wl.pages_needed(cfg, L, growth_tokens=cfg.n_steps) + 64
    max_bp = (cfg.length_cap + cfg.n_steps) // 16 + 2
    fo = wl.free_order(cfg, num_pages)
    kw = dims(cfg, num_pages, max_bp)
    o, g = orc.OracleCache(free_order=fo, **kw), GpuEngine(free_order=fo, **kw)
    populate(cfg, [o, g], L)
    assert _digest(o.state()) == _digest(g.state())

    # ---- oracle pass: record a digest per call and sampled attention per step
    log, ref_attn = [], {}

    def o_hook(name, step, cache, extra):
        st = cache.state()
        log.append((name, step, _digest(st)))
        if name == "append":
            nA = int(st["n_active"][0])
            rows = _sample_rows(nA)
            act = st["active_handles"][:nA]
            ref_attn[step] = (rows, cache.attention(wl.query(cfg, step)[act], rows=rows))

    res_o = oracle_trace(o, targets=targets, step_kv=lambda s: wl.step_kv(cfg, s), n_steps=cfg.n_steps,
                         prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: wl.scores(cfg, e),
                         on_call=o_hook)

    # ---- GPU pass: same inputs, compare at every call
    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()

    pos = [0]
    worst = [0.0]

    def g_hook(name, step, cache, extra):
        if name == "attention":
            act, out = extra
            rows, ref = ref_attn[step]
            got = out[torch.as_tensor(rows, device="cuda")].cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got))
            worst[0] = max(worst[0], float(np.abs(got - ref).max()))
            return
        st, rc = cache.get_state(with_status=True)
        assert rc == 0, (name, step, rc)
        exp = log[pos[0]]
        assert (name, step) == exp[:2], (name, step, exp[:2])
        assert _digest(st) == exp[2], f"integer state differs after {name} at step {step}"
        pos[0] += 1

    res_g = gpu_trace(g.c, targets=targets, step_kv=lambda s: tuple(dev(x) for x in wl.step_kv(cfg, s)),
                      query=lambda s: dev(wl.query(cfg, s)), n_steps=cfg.n_steps, prune_every=cfg.prune_every,
                      prune_k=cfg.prune_k, scores=lambda e: torch.from_numpy(wl.scores(cfg, e)).cuda(),
                      on_call=g_hook)
    assert pos[0] == len(log)
    assert res_g["branch_steps"] == res_o["branch_steps"]
    np.testing.assert_array_equal(res_g["done_step"], res_o["done_step"])
    np.testing.assert_array_equal(res_g["active_per_step"], res_o["active_per_step"])
    assert worst[0] <= TOL[cfg.dtype], worst[0]
    st = g.state()
    check_invariants(st, pt=16, num_pages=num_pages, Nb=cfg.nb, max_req=cfg.n_requests)
    # every request ended by early stop or by running out of branches (Algorithm 1's last test)
    c, p = st["req_counters"][:, 0], st["req_counters"][:, 1]
    ended = st["prefix_refcnt"] == 0
    assert np.all(((c >= cfg.quota) | (c + p == cfg.nb))[ended])     # a request without branches is done
    assert np.all((c < cfg.quota)[~ended])                            # and one at its quota has none left
    if st["n_active"][0] == 0:
        assert st["free_top"][0] == num_pages
    assert np.all(p <= np.where(c == 0, cfg.nb // 2, cfg.nb - 1))
    kinds = {n for n, _, _ in log}
    assert {"append", "finish", "prune"} <= kinds
    print(f"{size}: {len(log)} calls, {res_g['branch_steps']} branch-steps, requests done by step "
          f"{res_g['done_step'].max()}, early-stopped requests {int(np.sum(c >= cfg.quota))}/{cfg.n_requests}, "
          f"max abs attention err {worst[0]:.3g}")


def test_device_driven_trace_ends_where_the_oracle_ends():
    """The loops that keep the step on the device (rows addressed by branch handle, completion by target
    length, nothing read back between pruning steps; enqueued call by call, or recorded once into a HIP
    graph and replayed) and the host-driven loop must all leave the cache exactly where the oracle's own step
    loop leaves its cache: whole integer state, branch-steps, the attention of what is left; at sampled steps
    the by-handle output rows of the active branches equal the oracle's attention and the other rows are
    untouched."""
    import torch
    from paper_2505_13326_amd.trace import run_trace, run_trace_device
    cfg = wl.scaled(wl.CONFIGS[3], n_requests=5, length_params=(150, 0.8), length_cap=1200, n_steps=130, prune_every=20)
    L = wl.lengths(cfg)
    targets = (L + wl.remaining_tokens(cfg)).reshape(-1)
    num_pages = wl.pages_needed(cfg, L, growth_tokens=cfg.n_steps) + 64
    kw = dims(cfg, num_pages, (cfg.length_cap + cfg.n_steps) // 16 + 2)
    fo = wl.free_order(cfg, num_pages)

    o = orc.OracleCache(free_order=fo, **kw)
    populate(cfg, [o], L)
    res_o = oracle_trace(o, targets=targets, step_kv=lambda s: wl.step_kv(cfg, s), n_steps=cfg.n_steps,
                         prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: wl.scores(cfg, e),
                         query=lambda s: wl.query(cfg, s))
    want = (res_o["branch_steps"], _digest(o.state()))
    busy = int(np.sum(res_o["active_per_step"] > 0))

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()

    kvs = {s: tuple(dev(x) for x in wl.step_kv(cfg, s)) for s in range(1, cfg.n_steps + 1)}
    qs = {s: dev(wl.query(cfg, s)) for s in range(1, cfg.n_steps + 1)}
    args = dict(targets=targets, step_kv=lambda s: kvs[s], query=lambda s: qs[s], n_steps=cfg.n_steps,
                prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: torch.from_numpy(wl.scores(cfg, e)).cuda())
    H = cfg.n_handles
    sentinel = 12345.0
    for name, loop, extra in (("host", run_trace, {}), ("device", run_trace_device, {"graph": False}),
                              ("device, graph", run_trace_device, {"graph": True})):
        g = GpuEngine(free_order=fo, **kw)
        populate(cfg, [g], L)
        worst = [0.0]
        if loop is run_trace_device:
            out = torch.full((H, cfg.n_q_heads, cfg.head_dim), sentinel, dtype=torch.float32, device="cuda")

            def on_step(s, cache, o_dev):
                if s % 7 == 0:
                    o_dev.fill_(sentinel)                       # before the calls of a sampled step are enqueued
                if s % 7 != 1 or s not in res_o["outputs"]:
                    return
                act, ref = res_o["outputs"][s]
                got = o_dev.cpu().numpy()                       # waits for the step
                worst[0] = max(worst[0], float(np.abs(got[act].astype(np.float64) - ref).max()))
                rest = np.setdiff1d(np.arange(H), act)
                assert np.all(got[rest] == sentinel), "a row of a branch outside the batch was written"
            extra = dict(extra, out=out, on_step=on_step)
        res = loop(g.c, **args, **extra)
        st, rc = g.c.get_state(with_status=True)
        assert rc == 0
        assert (res["branch_steps"], _digest(st)) == want, name
        assert worst[0] <= TOL["bf16"], (name, worst[0])
        if loop is run_trace_device:
            assert busy <= res["steps_enqueued"] <= busy + cfg.prune_every, (name, busy, res["steps_enqueued"])
            assert g.c.active_count_hint() == int(st["n_active"][0])
        if int(st["n_active"][0]):                      # what is left attends alike on both sides
            compare_attention(cfg, o, g, wl.query(cfg, cfg.n_steps + 1))
        print(f"{name}: {res['branch_steps']} branch-steps, max abs by-handle attention err {worst[0]:.3g}, "
              f"steps enqueued {res.get('steps_enqueued', busy)} for {busy} with active branches")
