"""sart_decode_attention_static (the decode entry point that allocates nothing: its kernels' scratch
is a fixed array inside the library) against sart_decode_attention, through the C ABI: same bits, on
two calls in a row, the second over a smaller batch; then from a second cache of another geometry
(the array is shared by every call on the GPU and keeps the last call's contents); sizes beyond the
array are refused."""
import numpy as np
import pytest

import workloads as wl
from gpu_common import GpuEngine, dims, populate

pytestmark = pytest.mark.gpu


def _engine(shape, n_req, nb, P, med, seed_cfg=2, **kw):
    Hq, Hkv, d = shape
    cfg = wl.scaled(wl.CONFIGS[seed_cfg], n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_requests=n_req, nb=nb,
                    prompt_len=P, length_params=(med, 0.8), length_cap=4 * med)
    L = wl.lengths(cfg)
    g = GpuEngine(**dims(cfg, wl.pages_needed(cfg, L) + 8, int(-(-L.max() // 16)) + 2), **kw)
    populate(cfg, [g], L)
    return cfg, g


def _both_ways(cfg, g, step):
    """One decode through each entry point; returns the two outputs (the static one into a poisoned buffer)."""
    import torch
    st = g.state()
    act = st["active_handles"][:int(st["n_active"][0])]
    q = g.c._dev(wl.query(cfg, step)[act], (cfg.n_q_heads, cfg.head_dim))
    ref = g.c.decode_attention(q).clone()
    out = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    g.c.decode_attention(q, out=out, static_scratch=True)
    assert g.c.sync_status() == 0
    assert torch.isfinite(out).all()
    return ref, out


def test_static_scratch_decode_matches_the_allocating_entry_point():
    import torch
    import paper_2505_13326_amd as sart
    cfg, g = _engine((28, 4, 128), 4, 8, 200, 600)
    ref, out = _both_ways(cfg, g, 0)
    assert torch.equal(ref, out)                       # same kernels, same merge order: the same bits
    # second call, smaller input: drop three branches per request, append a token, decode again
    assert g.prune(sart.DROP_LOWEST_K, wl.scores(cfg, 0), k=3) == 0
    st = g.state()
    act = st["active_handles"][:int(st["n_active"][0])]
    assert len(act) == 4 * 5
    k, v = wl.step_kv(cfg, 1)
    assert g.append(sart.SEQ_BRANCH, None, None, k[act], v[act]) == 0
    ref2, out2 = _both_ways(cfg, g, 1)
    assert ref2.shape[0] == 20 and torch.equal(ref2, out2)
    # another cache, another geometry (natural layout: the generic kernel), then the first one again
    cfg3, g3 = _engine((8, 2, 64), 2, 3, 50, 100, force_natural_layout=True)
    ref3, out3 = _both_ways(cfg3, g3, 0)
    assert torch.equal(ref3, out3)
    ref4, out4 = _both_ways(cfg, g, 2)
    assert torch.equal(ref4, out4)


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    import paper_2505_13326_amd as sart
    # 4096 branches x 8 kv heads: a step may need more partial results than the array holds
    big = sart.SartCache(n_q_heads=40, n_kv_heads=8, head_dim=128, num_pages=64, max_requests=1024, branches_per_request=4,
                         max_pages_per_branch=2, max_prefix_pages=2, dtype="bf16")
    q = torch.zeros((4096, 40, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.full((4096, 40, 128), 3.0, dtype=torch.float32, device="cuda")
    with pytest.raises(sart.SartError) as e:
        big.decode_attention(q, out=out, static_scratch=True)
    assert e.value.status == sart.E_INVALID and "static scratch" in str(e.value)
    assert torch.all(out == 3.0) and big.sync_status() == 0
    # the same cache with a row buffer the array can serve is accepted (no active branch: nothing to write)
    big.decode_attention(q[:256], out=out[:256], static_scratch=True)
    assert big.sync_status() == 0 and torch.all(out == 3.0)
