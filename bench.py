#!/usr/bin/env python3
"""Benchmark of the SART decode hot path on one MI355X.

A step = one pass of the hot path over the batch: append one token of K/V to
every active branch (sart_append_tokens), then the decode attention of all
active branches (sart_decode_attention: partition, shared-prompt + private
split-K attention, merge).  Inputs are resident in HBM before timing starts.

The default run (--workload all) prints ONE JSON line whose top level is the
32B-like configuration (the benchmark's config 4, the largest single-GPU one),
with the 7B-like configuration (config 2) under "cfg2" and the early-stop /
prune trace (config 3, branch-steps/s over the whole 400-step loop) under
"cfg3"; each carries its own `roofline` (the attention kernel against the HBM
peak, and the whole sart_decode_attention call as decode_call_*) and
`cpu_baseline` (the float64 oracle on a stated sample).  --workload cfgN runs
one configuration alone.  prune / finish are timed once after the step loop
and reported in microseconds.  --gpus > 1 is refused: this build is
single-GPU by design.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# HBM traffic of the dominant kernel per launch: NOT measured in this run but copied from the rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE summary under profiles/ (k_attn_mfma_hbm_traffic_and_sq_counters.md), which states the
# commands; None = not measured for that workload
MEASURED_TRAFFIC_BYTES = {"cfg2": 1450971988, "cfg4": 10911881798}


def _request_arrays(wl, cfg, r, L):
    import numpy as np
    pk, pv = wl.prefix_kv(cfg, r)
    ids = [r * cfg.nb + j for j in range(cfg.nb)]
    ns = [int(L[r, j]) for j in range(cfg.nb)]
    kv = [wl.branch_kv(cfg, b, n) for b, n in zip(ids, ns)]
    return r, pk, pv, ids, ns, np.concatenate([x[0] for x in kv]), np.concatenate([x[1] for x in kv])


def mfma_probe_rates(sart, np, torch, shapes=((0, 512),), seconds=0.15):
    """What the matrix cores sustain on this machine on nothing but bf16 products from registers, for operands that
    are zero and operands drawn like the prompts' K/V (standard normal, rounded to bf16): the clock follows the
    power drawn and the power follows the operand values.  shapes: (product shape of sart_mfma_probe,
    workgroups) pairs; each is run for about `seconds` and the rate of the last launch is reported."""
    rng = np.random.default_rng(20250513)
    data = {"zeros": np.zeros(8192, np.float32), "normal_bf16": rng.standard_normal(8192).astype(np.float32)}
    rates = {}
    for shape, n_wg in shapes:
        sink = torch.empty(n_wg * 256, dtype=torch.float32, device="cuda")
        for name, host in data.items():
            ops = torch.from_numpy(host).to(torch.bfloat16).cuda()
            rounds, left, rate = 2000, seconds * 1e3, 0.0
            while left > 0:
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ev[0].record()
                sart.mfma_probe(ops, rounds, n_wg, sink, shape=shape)
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1])
                rate = n_wg * 4 * rounds * 524288.0 / (ms * 1e-3) / 1e12
                left -= ms
                rounds = max(2000, int(rounds * 25.0 / max(ms, 1e-3)))       # launches of about 25 ms
            key = f"{('32x32x16', '16x16x32', 'pair_loop_arithmetic')[shape]}_{n_wg // 256}_waves_per_simd_{name}"
            rates[key] = round(rate, 1)
    return rates


def bench_prefill(args, cfg, sart, wl, np, torch):
    """Prefill attention (Algorithm 1, Prefill) over the prompts of a configuration: one library call attends
    every request's whole prompt (causal).  The prompts' K/V are appended beforehand (not timed: they are the
    model's output, not this library's work).  value = algorithmic causal flops / time."""
    R, P = cfg.n_requests, cfg.prompt_len
    pp = -(-P // cfg.page_tokens)
    num_pages = R * pp + 8
    cache = sart.SartCache(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                           page_tokens=cfg.page_tokens, num_pages=num_pages, max_requests=R, branches_per_request=cfg.nb,
                           max_pages_per_branch=4, max_prefix_pages=pp,
                           dtype="fp8" if args.kv_dtype == "fp8" else cfg.dtype,
                           free_order=wl.free_order(cfg, num_pages) if args.free_order == "scattered" else None)

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()
    qs = []
    for r in range(R):
        k, v = wl.prefix_kv(cfg, r)
        qr = wl.prefix_query(cfg, r)
        if args.zero_data:                                   # what the operands' values cost: see --zero-data
            k, v, qr = np.zeros_like(k), np.zeros_like(v), np.zeros_like(qr)
        cache.append_tokens(sart.SEQ_PREFIX, [r], [P], k, v)
        qs.append(qr)
    q = dev(np.concatenate(qs))
    out = torch.empty((R * P, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    ids, nq = list(range(R)), [P] * R
    assert cache.sync_status() == 0
    K, W = args.steps, args.warmup
    for _ in range(W):
        cache.prefill_attention(ids, nq, q, out=out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for _ in range(K):
        cache.prefill_attention(ids, nq, q, out=out)
    ev[1].record()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / K
    k_ms = ev[0].elapsed_time(ev[1]) / K
    assert cache.sync_status() == 0
    flops = R * 4.0 * cfg.head_dim * cfg.n_q_heads * P * (P + 1) / 2
    kv_bytes = R * P * cfg.token_bytes
    roofline = {"bound": "mfma", "kernel": "k_prefill_b16" if cfg.dtype == "bf16" and args.kv_dtype != "fp8" else "k_prefill_mfma", "achieved": round(flops / (k_ms * 1e-3) / 1e12, 2),
                "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / (k_ms * 1e-3) / 1e12 / 2500.0, 4), "traffic": None,
                "algorithmic_flops_per_launch": int(flops), "kernel_ms_avg": round(k_ms, 4),
                "note": "events on the call's stream around all timed calls (validation kernel included)"}
    if cfg.dtype == "bf16" and args.kv_dtype != "fp8":
        # the kernel's own product shape and waves per SIMD: products alone, and with the softmax between them
        probe = mfma_probe_rates(sart, np, torch, shapes=((1, 512), (2, 512)))
        roofline["mfma_probe_tflops"] = probe
        roofline["frac_of_mfma_probe"] = round(roofline["achieved"] / probe["16x16x32_2_waves_per_simd_normal_bf16"], 4)
        roofline["frac_of_pair_loop_arithmetic"] = round(roofline["achieved"] / probe["pair_loop_arithmetic_2_waves_per_simd_normal_bf16"], 4)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as orc
        n = args.cpu_sample_requests or 1
        oc = orc.OracleCache(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                             page_tokens=cfg.page_tokens, num_pages=n * pp + 4, max_requests=R, branches_per_request=cfg.nb,
                             finish_quota=0, max_pages_per_branch=4, max_prefix_pages=pp, dtype=cfg.dtype)
        for r in range(n):
            k, v = wl.prefix_kv(cfg, r)
            assert oc.append(0, [r], [P], k, v) == 0
        t1 = time.perf_counter()
        for r in range(n):
            oc.prefill_attention(r, qs[r])
        dt_cpu = time.perf_counter() - t1
        cpu = {"value": round(n * flops / R / dt_cpu / 1e12, 5), "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"whole prompts of {n} of {R} requests, float64", "seconds": round(dt_cpu, 2)}
    return ({
        "metric": "prefill attention, algorithmic causal flops per second", "value": round(flops / dt / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(dt * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "all zero (measurement aid)" if args.zero_data else "synthetic",
        "config": {"workload": f"prompts of config {cfg.cfg_id}: {R} requests x {P} tokens, Hq {cfg.n_q_heads} / Hkv "
                               f"{cfg.n_kv_heads}, d {cfg.head_dim}, one call", "kv_bytes": kv_bytes},
        "roofline": roofline, "cpu_baseline": cpu})


def bench_trace(args, cfg, sart, wl, np, torch):
    """Config 3: the whole 400-step early-stop / prune loop (append + attention + finish + prune, host
    step loop included).  value = branch-decode-steps per second over the loop.  Returns the JSON record."""
    from paper_2505_13326_amd.trace import run_trace, run_trace_device
    L = wl.lengths(cfg)
    targets = (L + wl.remaining_tokens(cfg)).reshape(-1)
    num_pages = wl.pages_needed(cfg, L, growth_tokens=cfg.n_steps) + 64
    max_bp = (cfg.length_cap + cfg.n_steps) // 16 + 2

    def dev(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).cuda()

    kvs = [tuple(dev(x) for x in wl.step_kv(cfg, s)) for s in range(cfg.n_steps + 1)]
    qs = [dev(wl.query(cfg, s)) for s in range(cfg.n_steps + 1)]
    scs = [torch.from_numpy(wl.scores(cfg, e)).cuda() for e in range(cfg.n_steps // cfg.prune_every + 1)]
    out = torch.empty((cfg.n_handles, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    with ThreadPoolExecutor(max_workers=8) as ex:
        arrays = list(ex.map(lambda r: _request_arrays(wl, cfg, r, L), range(cfg.n_requests)))

    def new_cache():
        cache = sart.SartCache(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                               page_tokens=cfg.page_tokens, num_pages=num_pages, max_requests=cfg.n_requests,
                               branches_per_request=cfg.nb, finish_quota=cfg.quota, max_pages_per_branch=max_bp,
                               max_prefix_pages=cfg.prompt_len // cfg.page_tokens, dtype=cfg.dtype,
                               free_order=wl.free_order(cfg, num_pages))
        for r, pk, pv, ids, ns, bk, bv in arrays:
            cache.append_tokens(sart.SEQ_PREFIX, [r], [cfg.prompt_len], pk, pv)
            cache.append_tokens(sart.SEQ_BRANCH, ids, ns, bk, bv)
        assert cache.sync_status() == 0
        return cache

    times, res = [], None
    for rep in range(1 + max(1, min(args.steps, 3))):     # first repetition is the warm-up
        cache = new_cache()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if not args.host_loop:   # the step stays on the device: rows by handle, nothing read back between prunes
            res = run_trace_device(cache, targets=targets, step_kv=lambda s: kvs[s], query=lambda s: qs[s],
                                   n_steps=cfg.n_steps, prune_every=cfg.prune_every, prune_k=cfg.prune_k,
                                   scores=lambda e: scs[e], out=out, graph=args.graph)
        else:
            res = run_trace(cache, targets=targets, step_kv=lambda s: kvs[s], query=lambda s: qs[s], n_steps=cfg.n_steps,
                            prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: scs[e], out=out)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        assert cache.sync_status() == 0
        cache.close()
    dt = float(np.mean(times[1:]))
    busy = int(np.sum(res["active_per_step"] > 0)) if "active_per_step" in res else res["steps_enqueued"]

    # ---- the attention kernel's share of the loop: one more pass with HIP events around every step's kernel
    #      (each read waits for the device, so this pass is not the timed one) -------------------------------
    cache = new_cache()
    cache.set_profiling(1)
    k_ms, k_bytes = [], []

    def on_call(name, step, c, extra):
        if name != "attention":
            return
        a_ms, _ = c.last_decode_ms()
        st = c.get_state(fields=("n_active", "seq_lens", "prefix_refcnt"))
        n = int(st["n_active"][0])
        live = int(np.sum(st["prefix_refcnt"] > 0))
        k_ms.append(a_ms)
        k_bytes.append((int(st["seq_lens"][:n].sum()) + live * cfg.prompt_len) * cfg.token_bytes
                       + n * cfg.n_q_heads * cfg.head_dim * (cfg.elem_bytes + 4))
    run_trace(cache, targets=targets, step_kv=lambda s: kvs[s], query=lambda s: qs[s], n_steps=cfg.n_steps,
              prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: scs[e], out=out, on_call=on_call)
    cache.close()
    attn_s, attn_bytes = float(np.sum(k_ms)) * 1e-3, float(np.sum(k_bytes))
    roofline = {"bound": "hbm", "kernel": "k_attn_mfma", "achieved": round(attn_bytes / attn_s / 1e9, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(attn_bytes / attn_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                "algorithmic_bytes_all_launches": int(attn_bytes), "launches": len(k_ms), "kernel_ms_sum": round(attn_s * 1e3, 3),
                "kernel_ms_avg": round(attn_s * 1e3 / max(1, len(k_ms)), 4), "kernel_share_of_loop": round(attn_s / dt, 3),
                "note": "sum over the loop's attention launches (the batch shrinks from 256 to 0 branches): bytes / kernel time"}

    # ---- CPU baseline: the oracle's own loop on the same state, first steps only ---------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as orc
        from oracle.trace import run_trace as oracle_trace
        n_cpu_steps = 3
        oc = orc.OracleCache(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                             page_tokens=cfg.page_tokens, num_pages=num_pages, max_requests=cfg.n_requests,
                             branches_per_request=cfg.nb, finish_quota=cfg.quota, max_pages_per_branch=max_bp,
                             max_prefix_pages=cfg.prompt_len // cfg.page_tokens, dtype=cfg.dtype,
                             free_order=wl.free_order(cfg, num_pages))
        for r, pk, pv, ids, ns, bk, bv in arrays:
            assert oc.append(0, [r], [cfg.prompt_len], pk, pv) == 0
            assert oc.append(1, ids, ns, bk, bv) == 0
        t1 = time.perf_counter()
        ores = oracle_trace(oc, targets=targets, step_kv=lambda s: wl.step_kv(cfg, s), n_steps=n_cpu_steps,
                            prune_every=cfg.prune_every, prune_k=cfg.prune_k, scores=lambda e: wl.scores(cfg, e),
                            query=lambda s: wl.query(cfg, s))
        t_cpu = time.perf_counter() - t1
        cpu = {"value": round(ores["branch_steps"] / t_cpu, 2), "unit": "branch-steps/s", "cores": orc.num_threads(),
               "kind": "oracle", "sample": f"the oracle's own step loop (append, float64 attention of every active branch, "
               f"finish), steps 1..{n_cpu_steps} of {cfg.n_steps} ({ores['branch_steps']} branch-steps, {t_cpu:.2f} s wall, "
               "input generation included)"}
    return {
        "metric": "decode-attention achieved KV GB/s (fraction of HBM peak); branch-steps/s",
        "value": round(res["branch_steps"] / dt, 1), "unit": "branch-steps/s", "n_gpus": 1, "steps": cfg.n_steps,
        "warmup": 1, "ms_per_step": round(dt / max(1, busy) * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"cfg3 {cfg.name}: {cfg.n_requests} requests x {cfg.nb} branches, quota {cfg.quota}, "
                               f"{cfg.n_steps} steps, prune {cfg.prune_k} lowest every {cfg.prune_every} steps; whole "
                               "loop incl. host driver" + (", device-driven step (rows by handle, no state read back between prunes)"
                                                          + (" replayed from a HIP graph" if args.graph else "")
                                                          if not args.host_loop else ", host-driven step"), "branch_steps": res["branch_steps"],
                   "steps_with_active_branches": busy, "loop_s": round(dt, 4)},
        "roofline": roofline, "cpu_baseline": cpu}


def bench_probe_sweep(args, sart, np, torch):
    """What plain reads reach on this machine: the read probe (8 KiB chunks of a 2 GiB buffer) over workgroups,
    chunks in flight per wave, load flavour, chunk order and chunk-to-wave assignment.  One JSON line with
    the whole table (GB/s), best first."""
    nbytes = 1 << 31
    probe = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
    shuffled = torch.randperm(nbytes // 8192, device="cuda", dtype=torch.int32,
                              generator=torch.Generator(device="cuda").manual_seed(1))
    rows = []
    for order_name, od in (("sequential", None), ("shuffled", shuffled)):
        for inter in (0, 1):
            for flavour in (0, 1):
                for depth in (1, 2, 4, 8):
                    for wgs in (256, 512, 1024, 2048, 4096):
                        shape = (wgs, depth, flavour, inter)
                        for _ in range(2):
                            sart.read_probe(probe, od, shape=shape)
                        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                        ev[0].record()
                        for _ in range(args.steps if args.steps < 50 else 8):
                            sart.read_probe(probe, od, shape=shape)
                        ev[1].record()
                        torch.cuda.synchronize()
                        n = args.steps if args.steps < 50 else 8
                        rows.append({"order": order_name, "assignment": "interleaved" if inter else "contiguous",
                                     "loads": "non-temporal" if flavour else "plain", "chunks_in_flight": depth,
                                     "workgroups": wgs, "gbs": round(nbytes * n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9, 1)})
    rows.sort(key=lambda r: -r["gbs"])
    print(json.dumps({"metric": "plain read rate, 2 GiB buffer in 8 KiB chunks", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                      "best": rows[0], "table": rows}))


def bench_decode(args, cfg, workload, sart, wl, np, torch, K, W):
    """One configuration's step loop (append + decode attention), K timed steps after W warm-up steps.
    Returns the JSON record."""
    NL = max(1, args.layers)
    L = wl.lengths(cfg)
    growth = K + W + 2 * K + 64           # timed + profiled passes append one token per step
    num_pages = wl.pages_needed(cfg, L, growth_tokens=growth) + 64
    max_bp = (cfg.length_cap + growth) // cfg.page_tokens + 2
    fo = wl.free_order(cfg, num_pages) if args.free_order == "scattered" else None
    cache = sart.SartCache(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                           page_tokens=cfg.page_tokens, num_pages=num_pages, max_requests=cfg.n_requests,
                           branches_per_request=cfg.nb, finish_quota=cfg.quota, max_pages_per_branch=max_bp,
                           max_prefix_pages=max(1, cfg.prompt_len // cfg.page_tokens),
                           dtype="fp8" if args.kv_dtype == "fp8" else cfg.dtype, free_order=fo, n_layers=NL)
    if args.merge == "in-kernel":
        cache.set_merge_mode(True)
    if args.no_stagger:
        cache.set_prompt_stagger(False)
    if args.workgroups or args.prompt_mode >= 0 or args.skew is not None:
        cache.set_decode_launch(args.workgroups, args.prompt_mode, sart.DEFAULT_SKEW_PERMILLE if args.skew is None else args.skew)

    # ---- CPU baseline cache (oracle) on a bounded sample of the same workload ------------
    do_cpu = not args.no_cpu_baseline and args.kv_dtype == "bf16"     # the CPU baseline is timed on the bf16 cache
    n_cpu = args.cpu_sample_requests or {2: 16, 4: 4, 5: 1}[cfg.cfg_id]
    n_cpu = min(n_cpu, cfg.n_requests)
    ocache = None
    if do_cpu:
        import oracle as orc
        Ls = L[:n_cpu]
        ocache = orc.OracleCache(
            n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, page_tokens=cfg.page_tokens,
            num_pages=int(np.sum((Ls + 15) // 16)) + n_cpu * (cfg.prompt_len // 16 + 1) + 8, max_requests=cfg.n_requests,
            branches_per_request=cfg.nb, finish_quota=cfg.quota, max_pages_per_branch=max_bp,
            max_prefix_pages=max(1, cfg.prompt_len // cfg.page_tokens), dtype=cfg.dtype)

    t0 = time.time()
    with ThreadPoolExecutor(max_workers=8) as ex:
        for r, pk, pv, ids, ns, bk, bv in ex.map(lambda r: _request_arrays(wl, cfg, r, L), range(cfg.n_requests)):
            if NL == 1:
                cache.append_tokens(sart.SEQ_PREFIX, [r], [cfg.prompt_len], pk, pv)
                cache.append_tokens(sart.SEQ_BRANCH, ids, ns, bk, bv)
            else:   # every layer gets the same values (uploaded once): the timing does not depend on them
                dpk, dpv, dbk, dbv = (cache._dev(x, (cfg.n_kv_heads, cfg.head_dim)) for x in (pk, pv, bk, bv))
                for l in range(NL):
                    cache.append_tokens(sart.SEQ_PREFIX, [r], [cfg.prompt_len], dpk, dpv, layer=l)
                for l in range(NL):
                    cache.append_tokens(sart.SEQ_BRANCH, ids, ns, dbk, dbv, layer=l)
            if ocache is not None and r < n_cpu:
                assert ocache.append(0, [r], [cfg.prompt_len], pk, pv) == 0
                assert ocache.append(1, ids, ns, bk, bv) == 0
    assert cache.sync_status() == 0
    st = cache.get_state()
    nA = int(st["n_active"][0])
    assert nA == cfg.n_handles
    t_build = time.time() - t0

    # ---- per-step inputs, resident on the device --------------------------------------
    def dev(x):
        t = torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16) if cfg.dtype == "bf16" \
            else torch.from_numpy(np.ascontiguousarray(x))
        return t.cuda()
    n_in = 4
    qs = [dev(wl.query(cfg, s)) for s in range(n_in)]
    kvs = [tuple(dev(x) for x in wl.step_kv(cfg, s)) for s in range(n_in)]
    out = torch.empty((nA, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")

    def step(i):
        k, v = kvs[i % n_in]
        for l in range(NL):          # a model's forward: every layer appends its K/V of the token, then attends
            cache.append_tokens(sart.SEQ_BRANCH, None, None, k, v, layer=l)
            cache.decode_attention(qs[i % n_in], out=out, layer=l)

    if args.graph:
        # the step (all-active append + attention) recorded once per input set and replayed
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        def graph_body(j):
            for l in range(NL):
                cache.append_tokens(sart.SEQ_BRANCH, None, None, kvs[j][0], kvs[j][1], all_active=True, layer=l)
                cache.decode_attention(qs[j], out=out, layer=l)
        with torch.cuda.stream(side):
            graph_body(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs = []
        for j in range(n_in):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                graph_body(j)
            graphs.append(gr)

        def step(i):
            graphs[i % n_in].replay()

    def tokens_now():
        s = cache.get_state()
        n = int(s["n_active"][0])
        return int(s["seq_lens"][:n].sum()), cfg.n_requests * cfg.prompt_len

    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    priv0, pre = tokens_now()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert cache.sync_status() == 0
    ms_step = dt / K * 1e3
    # private tokens read at timed step i (1-based): priv0 + i*nA
    mean_tokens = priv0 + nA * (K + 1) / 2 + pre
    tok_bytes = cfg.token_bytes // (2 if args.kv_dtype == "fp8" else 1)     # an 8-bit float cache keeps half the bytes
    kv_bytes = mean_tokens * tok_bytes
    io_bytes = nA * cfg.n_q_heads * cfg.head_dim * (cfg.elem_bytes + 4)     # q read + out write
    alg_bytes = kv_bytes + io_bytes
    logical_bytes = (priv0 + nA * (K + 1) / 2 + nA * cfg.prompt_len) * tok_bytes
    value = NL * kv_bytes / (dt / K) / 1e9

    # ---- dominant kernel timed with HIP events on its own stream -----------------------
    cache.set_profiling(args.kernel_repeats)
    attn_ms, total_ms = [], []
    priv1, _ = tokens_now()
    n_prof = max(1, K // max(1, args.kernel_repeats // 2))
    for i in range(n_prof):
        (eager_step if args.graph else step)(i)      # the event-timed pass launches eagerly
        a, t = cache.last_decode_ms()
        attn_ms.append(a)
        total_ms.append(t)
    cache.set_profiling(0)
    attn_avg = float(np.mean(attn_ms))
    alg_bytes_prof = (priv1 + nA * (n_prof + 1) / 2 + pre) * tok_bytes + io_bytes
    achieved = alg_bytes_prof / (attn_avg * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_attn_mfma", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(workload) if args.kv_dtype == "bf16" else None,
                "algorithmic_bytes_per_launch": int(alg_bytes_prof), "kernel_ms_avg": round(attn_avg, 4),
                "kernel_ms_p10_p50_p90": [round(float(np.percentile(attn_ms, p)), 4) for p in (10, 50, 90)],
                "launches_per_event_pair": args.kernel_repeats}
    # the whole sart_decode_attention call (attention kernel + merge), back to back without appends, wall clock
    n_call = max(10, K // 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_call):
        cache.decode_attention(qs[i % n_in], out=out)
    torch.cuda.synchronize()
    call_ms = (time.perf_counter() - t0) / n_call * 1e3
    priv2, _ = tokens_now()
    call_bytes = (priv2 + pre) * tok_bytes + io_bytes
    roofline["decode_call_ms_avg"] = round(call_ms, 4)
    roofline["decode_call_frac"] = round(call_bytes / (call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)

    # ---- what plain reads reach on this machine: 8 KiB chunks of a 2 GiB buffer, in order and shuffled, with ordinary
    #      loads and with the non-temporal hint the attention kernel's own-page loads carry (the best launch
    #      shapes of `--workload probe`, profiles/read_probe_sweep.md) ------------------------------------------
    probe = torch.ones(1 << 31, dtype=torch.uint8, device="cuda")
    order = torch.randperm((1 << 31) // 8192, device="cuda", dtype=torch.int32, generator=torch.Generator(device="cuda").manual_seed(1))
    rates = {}
    for name, od, shape in (("sequential", None, None), ("shuffled_8KiB", order, None),
                            ("sequential_nontemporal", None, (256, 1, 1, 1)), ("shuffled_8KiB_nontemporal", order, (2048, 4, 1, 0))):
        for _ in range(3):
            sart.read_probe(probe, od, shape=shape)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        evs[0].record()
        for _ in range(10):
            sart.read_probe(probe, od, shape=shape)
        evs[1].record()
        torch.cuda.synchronize()
        rates[name] = round((1 << 31) * 10 / (evs[0].elapsed_time(evs[1]) * 1e-3) / 1e9, 1)
    del probe, order
    roofline["read_probe_gbs"] = rates
    roofline["frac_of_read_probe"] = round(achieved / rates["shuffled_8KiB_nontemporal"], 4)

    # ---- maintenance calls, once each (they change the batch, so after the step loop) --
    sc = torch.from_numpy(wl.scores(cfg, 0)).cuda()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cache.prune_branches(sart.DROP_LOWEST_K, sc, k=1)
    torch.cuda.synchronize()
    prune_us = (time.perf_counter() - t0) * 1e6
    s2 = cache.get_state()
    n2 = int(s2["n_active"][0])
    fin = s2["active_handles"][:n2][::max(1, cfg.nb - 1)][:cfg.n_requests]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cache.finish_branch(fin)
    torch.cuda.synchronize()
    finish_us = (time.perf_counter() - t0) * 1e6
    assert cache.sync_status() == 0

    # ---- CPU baseline: the oracle as it stands, same workload (bounded sample) ---------
    cpu = None
    if do_cpu:
        import oracle as orc
        so = ocache.state()
        nO = int(so["n_active"][0])
        act = so["active_handles"][:nO]
        q0 = wl.query(cfg, 0)[act]
        # the same decode step over again until about a second has passed (some 10-20 s of CPU work on the
        # box's 16 threads)
        reps, t0 = 0, time.perf_counter()
        while True:
            ocache.attention(q0)
            reps += 1
            t_all = time.perf_counter() - t0
            if t_all >= 1.0 or reps >= 64:
                break
        t_cpu = t_all / reps
        o_bytes = (int(so["seq_lens"][:nO].sum()) + n_cpu * cfg.prompt_len) * cfg.token_bytes
        cpu = {"value": round(o_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"float64 oracle attention of requests 0..{n_cpu - 1} of {cfg.n_requests} "
                         f"({nO} branches, {o_bytes / 1e6:.0f} MB of KV per decode step; {reps} steps in {t_all:.2f} s wall)",
               "branch_steps_per_s": round(nO / t_cpu, 2)}

    line = {
        "metric": "decode-attention achieved KV GB/s (fraction of HBM peak); branch-steps/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype if args.kv_dtype == "bf16" else "bf16 arithmetic on an fp8 (E4M3) cache", "data": "synthetic",
        "config": {"workload": f"{workload} {cfg.name}: {cfg.n_requests} requests x {cfg.nb} branches, "
                               f"Hq{cfg.n_q_heads}/Hkv{cfg.n_kv_heads} d{cfg.head_dim} {cfg.dtype if args.kv_dtype == 'bf16' else 'fp8 cache'}, prompt "
                               f"{cfg.prompt_len}, private lengths {cfg.length_dist}{cfg.length_params} cap "
                               f"{cfg.length_cap}, page 16, free order {args.free_order}",
                   "active_branches": nA, "layers": NL, "kv_bytes_per_step": int(NL * kv_bytes),
                   "step": "append 1 token/branch + decode attention" + (f", for each of {NL} layers" if NL > 1 else "")},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "branch_steps_per_s": round(nA / (dt / K), 1),
        "logical_kv_gbs": round(logical_bytes / (dt / K) / 1e9, 1),
        "prune_us": round(prune_us, 1), "finish_us": round(finish_us, 1),
        "build_state_s": round(t_build, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    cache.close()
    if ocache is not None:
        ocache.close()
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all", choices=["all", "cfg2", "cfg3", "cfg4", "cfg5", "copy", "probe", "mfma_probe", "prefill4", "prefill5"],
                    help="all = config 4 (the headline) with configs 2 and 3 nested in the same line; copy = a plain 1 GiB device copy, the known-size kernel that calibrates the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters; prefillN = prefill attention over the prompts "
                         "of config N")
    ap.add_argument("--free-order", default="scattered", choices=["scattered", "identity"])
    ap.add_argument("--workgroups", type=int, default=0, help="attention workgroups (0 = library default)")
    ap.add_argument("--prompt-mode", type=int, default=-1, help="0 = chosen per step by the library (default), 1 = prompt blocks read by every branch, 2 = prompt blocks read once for a tile of 16 of a request's query rows, -1 = library default")
    ap.add_argument("--skew", type=int, default=None, help="per-mille of work moved from odd to even workgroups (default: library's)")
    ap.add_argument("--prompt-len", type=int, default=-1, help="override the workload's prompt length (experiments)")
    ap.add_argument("--requests", type=int, default=-1, help="override the workload's number of requests (experiments)")
    ap.add_argument("--kernel-repeats", type=int, default=8,
                    help="launches of the attention kernel between the two HIP events of the profiled pass")
    ap.add_argument("--kv-dtype", default="bf16", choices=["bf16", "fp8"], help="fp8: the cache keeps K and V as 8-bit floats "
                    "(E4M3; bf16 crosses the boundary): half the bytes per cached token")
    ap.add_argument("--layers", type=int, default=1, help="layers sharing the tables; a step appends to and attends over "
                    "every layer (same values in every layer)")
    ap.add_argument("--merge", default="kernel", choices=["in-kernel", "kernel"], help="where a step's partial results "
                    "are merged: by the separate merge kernel (default) or by the attention kernel's last writers")
    ap.add_argument("--no-stagger", action="store_true", help="every wave serves its prompt work before its own range")
    ap.add_argument("--graph", action="store_true", help="replay the step (append + attention) from a HIP graph (cfg3: the device-driven step)")
    ap.add_argument("--host-loop", action="store_true", help="cfg3: the host-driven step (the host gathers the active rows and lists the completed "
                    "branches, reading the state back after every call that changes the batch) instead of the device-driven one")
    ap.add_argument("--zero-data", action="store_true", help="prefill workloads: all-zero Q, K and V instead of the seeded draws "
                    "(the matrix cores' clock follows the power drawn, and that the operand values: a measurement aid, not a result)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-requests", type=int, default=0, help="requests the oracle is timed on (0 = auto)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (requests are independent and would shard with no "
              "collective); --gpus > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_13326_amd as sart
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload == "copy":
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.warmup):
            dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"metric": "device copy", "bytes_read": n, "bytes_written": n, "steps": args.steps,
                          "ms_per_step": round(dt * 1e3, 4), "value": round(2 * n / dt / 1e9, 1), "unit": "GB/s"}))
        return
    if args.workload == "probe":
        return bench_probe_sweep(args, sart, np, torch)
    if args.workload == "mfma_probe":
        print(json.dumps({"metric": "bf16 matrix-core products from registers and nothing else, by product shape and waves per SIMD",
                          "unit": "TFLOP/s", "value": mfma_probe_rates(sart, np, torch, shapes=((0, 512), (0, 256), (1, 512), (1, 256), (2, 512), (2, 256)), seconds=0.8),
                          "peak": 2500.0}))
        return
    if args.workload == "all":
        # the headline: config 4 (largest single-GPU configuration), with config 2 and the config 3 trace nested
        line = bench_decode(args, wl.CONFIGS[4], "cfg4", sart, wl, np, torch, args.steps, args.warmup)
        torch.cuda.empty_cache()
        keep = ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "frac_of_hbm_peak", "branch_steps_per_s",
                "logical_kv_gbs", "prune_us", "finish_us", "roofline", "cpu_baseline")
        sub = bench_decode(args, wl.CONFIGS[2], "cfg2", sart, wl, np, torch, max(args.steps, 50), max(args.warmup, 10))
        line["cfg2"] = {k: sub[k] for k in keep}
        torch.cuda.empty_cache()
        sub = bench_trace(args, wl.CONFIGS[3], sart, wl, np, torch)
        line["cfg3"] = {k: sub[k] for k in keep if k in sub}
        torch.cuda.empty_cache()
        # Algorithm 1's Prefill over config 4's prompts (a dense contraction: held against the matrix-core peak)
        args.steps, args.warmup = 20, 3
        sub = bench_prefill(args, wl.CONFIGS[4], sart, wl, np, torch)
        line["prefill4"] = {k: sub[k] for k in keep if k in sub}
        print(json.dumps(line), flush=True)
        return
    cfg = wl.CONFIGS[int(args.workload[-1])]
    if args.prompt_len >= 0:
        cfg = wl.scaled(cfg, prompt_len=args.prompt_len)
    if args.requests > 0:
        cfg = wl.scaled(cfg, n_requests=args.requests)
    if args.workload.startswith("prefill"):
        print(json.dumps(bench_prefill(args, cfg, sart, wl, np, torch)), flush=True)
        return
    if cfg.cfg_id == 3:
        print(json.dumps(bench_trace(args, cfg, sart, wl, np, torch)), flush=True)
        return
    print(json.dumps(bench_decode(args, cfg, args.workload, sart, wl, np, torch, args.steps, args.warmup)), flush=True)


if __name__ == "__main__":
    main()
