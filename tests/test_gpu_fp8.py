"""8-bit float (E4M3) KV cache on the GPU against the oracle: every stored code,
decode attention and prefill attention, small shapes and the 7B-like size."""
import numpy as np
import pytest

import oracle as orc
import workloads as wl
from gpu_common import GpuEngine, compare_attention, dims, populate
from helpers import assert_state_equal

pytestmark = pytest.mark.gpu

TOL_FP8 = 1e-2      # bf16 arithmetic on exactly expanded codes: the bf16 bound of the benchmark spec


def _kw(cfg, pages, max_bp, max_pp=None, **extra):
    kw = dims(cfg, pages, max_bp, max_pp=max_pp)
    kw["dtype"] = "fp8"
    kw.update(extra)
    return kw


def _k_byte(d_dim, token, d):      # the header's MFMA16_FP8 layout, retyped
    return ((d // 64) * 64 + ((d // 8) % 4) * 16 + token) * 16 + 8 * ((d // 32) % 2) + d % 8


def _v_byte(d_dim, token, d):
    return ((d // 64) * 64 + (token // 4) * 16 + d % 16) * 16 + 8 * ((d // 32) % 2) + 4 * ((d // 16) % 2) + token % 4


@pytest.mark.parametrize("scale", [1.0, 0.37])
def test_every_bf16_value_is_stored_as_the_oracles_code(scale):
    import torch
    Hkv, d = 2, 64
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits = bits[np.isfinite(wl.bf16_bits_to_f32(bits))]
    per_tok = Hkv * d
    n_tok = -(-bits.size // per_tok)
    pad = np.zeros(n_tok * per_tok, np.uint16)
    pad[:bits.size] = bits
    k = pad.reshape(n_tok, Hkv, d)
    v = k[::-1].copy()                                           # V gets the values in another order
    pages = n_tok // 16 + 2
    pool = torch.zeros(pages * 16 * 2 * Hkv * d, dtype=torch.uint8, device="cuda")
    import paper_2505_13326_amd as sart
    c = sart.SartCache(n_q_heads=4, n_kv_heads=Hkv, head_dim=d, num_pages=pages, max_requests=1, branches_per_request=1,
                       max_pages_per_branch=1, max_prefix_pages=pages, dtype="fp8", kv_pool=pool, k_scale=scale,
                       v_scale=scale)
    assert c.layout == sart.LAYOUT_MFMA16_FP8
    c.append_tokens(sart.SEQ_PREFIX, [0], [n_tok], k, v)
    assert c.sync_status() == 0
    raw = pool.cpu().numpy()
    table = c.get_state()["prefix_tables"][0]
    want_k, _ = orc.fp8_roundtrip(k, scale)
    want_v, _ = orc.fp8_roundtrip(v, scale)
    tile = 16 * d
    tok = np.arange(n_tok)
    page_base = table[tok // 16].astype(np.int64) * (Hkv * 2 * tile)
    for h in range(Hkv):
        for dd in range(d):
            kb = page_base + h * 2 * tile + np.array([_k_byte(d, int(t % 16), dd) for t in tok])
            vb = page_base + h * 2 * tile + tile + np.array([_v_byte(d, int(t % 16), dd) for t in tok])
            # +0 and -0 are one value
            gk, gv = raw[kb], raw[vb]
            wk, wv = want_k[:, h, dd], want_v[:, h, dd]
            assert np.all((gk == wk) | (((gk | wk) & 0x7f) == 0)), (h, dd)
            assert np.all((gv == wv) | (((gv | wv) & 0x7f) == 0)), (h, dd)


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.5, 0.25), (0.37, 1.7)], ids=["unit", "pow2", "free"])
@pytest.mark.parametrize("shape", [(28, 4, 128), (40, 8, 128), (8, 2, 64), (16, 1, 128)], ids=["g7", "g5", "g4d64", "g16"])
def test_fp8_decode_and_prefill_small(shape, scales):
    Hq, Hkv, d = shape
    ks, vs = scales
    cfg = wl.scaled(wl.CONFIGS[2], n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_requests=3, nb=5, prompt_len=100,
                    length_params=(200, 0.8), length_cap=1500)
    L = wl.lengths(cfg)
    L[0, 0], L[0, 1], L[1, 0] = 1, 16, 17
    pages = wl.pages_needed(cfg, L) + 4
    kw = _kw(cfg, pages, int(-(-L.max() // 16)) + 1, free_order=wl.free_order(cfg, pages), k_scale=ks, v_scale=vs)
    o = orc.OracleCache(**kw)
    g = GpuEngine(**kw)
    populate(cfg, [o, g], L)
    assert_state_equal(o.state(), g.state())
    err = compare_attention(cfg, o, g, wl.query(cfg, 0), tol=TOL_FP8)
    # one decode step, other launch shapes
    st = o.state()
    act = st["active_handles"][:int(st["n_active"][0])]
    k, v = wl.step_kv(cfg, 1)
    for e in (o, g):
        assert e.append(orc.SEQ_BRANCH, None, None, k[act], v[act]) == orc.OK
    for n_wg, pmode in ((3, 1), (64, 2), (256, 1), (256, 2)):      # prompt blocks per branch / shared by the request's rows
        g.c.set_decode_launch(n_wg, pmode, 50)
        compare_attention(cfg, o, g, wl.query(cfg, 1), tol=TOL_FP8)
    # prefill over the same prompts
    q = wl.prefix_query(cfg, 1)
    got = g.c.prefill_attention([1], [cfg.prompt_len], q).cpu().numpy().astype(np.float64)
    perr = float(np.abs(got - o.prefill_attention(1, q)).max())
    assert perr <= TOL_FP8
    print(f"fp8 {shape} scales {scales}: decode max abs err {err:.3g}, prefill {perr:.3g}")


def test_fp8_rejects_shapes_without_the_tile():
    import paper_2505_13326_amd as sart
    with pytest.raises(sart.SartError):
        sart.SartCache(n_q_heads=4, n_kv_heads=1, head_dim=96, num_pages=8, max_requests=1, branches_per_request=1,
                       max_pages_per_branch=2, max_prefix_pages=2, dtype="fp8")
    with pytest.raises(sart.SartError):
        sart.SartCache(n_q_heads=4, n_kv_heads=1, head_dim=128, page_tokens=8, num_pages=8, max_requests=1,
                       branches_per_request=1, max_pages_per_branch=2, max_prefix_pages=2, dtype="fp8")


def test_fp8_7b_like_full_size_sampled():
    cfg = wl.CONFIGS[2]
    L = wl.lengths(cfg)
    reqs = [0, 5, 11]
    pages = int(np.sum((L[reqs] + 15) // 16)) + len(reqs) * 32 + 8
    kw = _kw(cfg, pages, cfg.length_cap // 16 + 2, free_order=wl.free_order(cfg, pages))
    o = orc.OracleCache(**kw)
    g = GpuEngine(**kw)
    populate(cfg, [o, g], L, requests=reqs)
    assert_state_equal(o.state(), g.state())
    nA = int(o.state()["n_active"][0])
    rows = sorted(set(np.random.default_rng(5).integers(0, nA, size=6).tolist() + [0, nA - 1]))
    err = compare_attention(cfg, o, g, wl.query(cfg, 0), rows=rows, tol=TOL_FP8)
    print(f"fp8 config 2 (3 requests): max abs err {err:.3g}")
